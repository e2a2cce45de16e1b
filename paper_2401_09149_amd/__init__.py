"""MI355X-native exact causal attention (forward and backward) for long-sequence training.

The HIP library is loaded on first use by `paper_2401_09149_amd.binding`; importing the
package itself touches neither the GPU nor the shared library.
"""
