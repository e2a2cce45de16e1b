/*
 * ie_linear — the Linear modules of a Transformer layer without bias, forward and backward, in bf16 with
 * fp32 accumulation on the matrix cores (MI355X / gfx950).
 *
 * Next to self-attention the linear modules are the main contributors to a layer's computation time, and
 * under sequence parallelism without tensor parallelism each GPU applies them to its (b, S/s_sp, H) slice
 * of the input with the complete weight matrices (Sec. 2.4 "SP-2"; Sec. 4.2 "Computation Profiler").  With
 * M = b * S/s_sp tokens, weight w [N, K] (N outputs, K inputs, as stored by the framework):
 *     forward          y  = x w^T        x  [M, K] -> y  [M, N]
 *     backward, input  dx = dy w         dy [M, N] -> dx [M, K]
 *     backward, weight dw = dy^T x       dy [M, N], x [M, K] -> dw [N, K]
 * All tensors are contiguous row-major bf16; products accumulate in fp32 and are rounded to bf16 (nearest
 * even) once, on output.  dw is the gradient of this call's tokens only: it is overwritten, not
 * accumulated into.
 *
 * Conventions: as in ie_attn.h (device pointers owned by the caller, work enqueued on `stream`, no host
 * synchronisation, no allocation, status codes of ie_attn_status).  Every pointer must be 16-byte aligned
 * (IE_ERR_ALIGN).  Supported (IE_ERR_UNSUPPORTED otherwise): the contracted dimension (K forward, N for dx, M
 * for dw) a multiple of 64, the other dimensions that are contiguous in memory (N and K) multiples of 8; M is
 * otherwise arbitrary.  Dimensions must be positive, N and K below 2^22 (IE_ERR_SHAPE).  On error nothing has
 * been launched, except for IE_ERR_HIP.
 */
#ifndef IE_LINEAR_H
#define IE_LINEAR_H

#include "ie_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* y[M,N] = x[M,K] w[N,K]^T (Sec. 2.1: the linear modules of the attention and MLP blocks; Sec. 4.2). */
int ie_linear_fwd(const void* x, const void* w, void* y, int64_t M, int64_t N, int64_t K, void* stream);

/* dx[M,K] = dy[M,N] w[N,K]: gradient with respect to the module's input. */
int ie_linear_bwd_input(const void* dy, const void* w, void* dx, int64_t M, int64_t N, int64_t K, void* stream);

/* dw[N,K] = dy[M,N]^T x[M,K]: gradient with respect to the weight (the appendix "Implementation Detail: Selective Overlap": backward costs about twice the
 * forward: two products instead of one). */
int ie_linear_bwd_weight(const void* dy, const void* x, void* dw, int64_t M, int64_t N, int64_t K, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* IE_LINEAR_H */
