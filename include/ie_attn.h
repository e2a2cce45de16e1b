/*
 * ie_attn — exact softmax attention, forward and backward, for one GPU's share of the
 * heads over the full sequence (MI355X / gfx950).
 *
 * This is the per-GPU step of hybrid sequence parallelism: after the first all-to-all
 * every GPU holds Q, K and V of all S tokens for heads/s_sp heads, laid out
 * [B, S, heads_local, head_dim] (Sec. 2.4 "SP-2", Sec. 3.2.2 "Sequence Parallelism"), and
 * runs fused multi-head attention on them (Sec. 2.1 "Transformer Architecture";
 * Sec. 4.2 "Computation Profiler": self-atten(b, S, H, D/s_sp) on a single GPU).  The
 * backward pass recomputes the probabilities instead of storing them (Sec. 3.2: the
 * fused kernel includes selective activation recomputation), so only o and the
 * per-row log-sum-exp travel from forward to backward.
 *
 * Definition (batch b, query head h, kv head g = h / (Hq/Hkv), token i in document
 * [a, e); the visible keys are a <= j <= i when causal, a <= j < e otherwise):
 *     s_ij  = scale * <q[b,i,h,:], k[b,j,g,:]>
 *     lse_i = ln sum_j exp(s_ij)            p_ij = exp(s_ij - lse_i)
 *     o[b,i,h,:] = sum_j p_ij v[b,j,g,:]
 *     delta_i = <dout[b,i,h,:], o[b,i,h,:]>     ds_ij = p_ij (<dout_i, v_j> - delta_i)
 *     dq_i = scale sum_j ds_ij k_j
 *     dk_j = scale sum_{h in group g} sum_i ds_ij q_i      dv_j = sum_{h in g} sum_i p_ij dout_i
 *
 * Common conventions
 *   - Every pointer is a DEVICE pointer on the current HIP device; the caller owns all
 *     buffers.  The library allocates no device memory and never synchronises with the host: all
 *     work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default
 *     stream) and the buffers must stay alive until the stream has passed it.
 *     Calls may overlap on different streams.  The main kernels are persistent and draw their work from a few
 *     counters per launch.  The backward kernels keep them in the caller's workspace, where the call's first
 *     kernel clears them: two backward calls that overlap must not share a workspace.  ie_attn_fwd (head
 *     dimension 128, 256-row items) takes them from 256 slots of a device array inside the library, which
 *     every launch leaves cleared; a slot is handed out again only when the event recorded behind its
 *     previous launch has completed, or to a launch on the same stream, and when every slot is in flight on
 *     other streams the call returns IE_ERR_BUSY rather than share one.
 *     A call enqueues kernel launches only (no memset, no copy, no allocation), so it may be recorded
 *     under stream capture; a forward call captured into a graph keeps its counter slot for the life of
 *     the process (at most 256 such calls), and two replays of one graph must not run at the same time.
 *   - q, o, dout, dq : contiguous [B, S, Hq,  D] bf16.
 *     k, v, dk, dv   : contiguous [B, S, Hkv, D] bf16.
 *     lse            : contiguous [B, Hq, S] fp32, natural log, `scale` included.
 *   - bf16 outputs are rounded to nearest even from fp32 accumulators.
 *   - Packed documents: cu_seqlens != NULL is an int32 device array of num_docs+1
 *     non-decreasing offsets with cu_seqlens[0] = 0 and cu_seqlens[num_docs] = S; B must
 *     be 1; tokens attend only inside their own document (block-diagonal mask);
 *     empty documents are allowed.  The array's contents are not read on the host and
 *     are therefore not validated; offsets outside [0, S] give undefined results.
 *     cu_seqlens == NULL (num_docs ignored) means one document per batch entry.
 *   - Supported: D in {64, 128}; Hq % Hkv == 0; scale finite and > 0; causal in {0, 1};
 *     any S >= 1 with B*S*Hq*D < 2^40 elements.
 *   - Return value: 0 on success or a negative ie_attn_status; nothing is printed and
 *     no exception crosses the boundary.  On error no kernel has been launched, except
 *     for IE_ERR_HIP, which reports a failed launch part-way through a call.
 */
#ifndef IE_ATTN_H
#define IE_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ie_attn_status {
  IE_OK = 0,
  IE_ERR_NULL = -1,        /* a required pointer is NULL */
  IE_ERR_SHAPE = -2,       /* B, S, Hq, Hkv <= 0; Hq % Hkv != 0; packed with B != 1 or num_docs < 1; size too large */
  IE_ERR_UNSUPPORTED = -3, /* D not in {64,128}; scale not finite or <= 0; causal not 0/1 */
  IE_ERR_WORKSPACE = -4,   /* workspace NULL, misaligned (256 B) or smaller than ie_attn_bwd_workspace_bytes */
  IE_ERR_HIP = -5,         /* a HIP call failed; ie_attn_last_hip_error() has the runtime's text */
  IE_ERR_ALIGN = -6,       /* a pointer is not 16-byte aligned (ie_sp.h) */
  IE_ERR_BUSY = -7         /* ie_attn_fwd: all work-queue slots are in flight or held by captured graphs (see above) */
} ie_attn_status;

/*
 * Forward: writes o and lse for every token (steps "S = QK^T, mask, online softmax,
 * O = PV" of fused attention; Sec. 2.1, Sec. 4.2).  Both outputs are fully overwritten.
 */
int ie_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                const int32_t* cu_seqlens, int32_t num_docs,
                int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D,
                float scale, int32_t causal, void* stream);

/*
 * Bytes of device workspace ie_attn_bwd needs for this shape: 8 * B * Hq * S (rounded up) + 256.  It holds -delta and
 * -lse * log2(e), [B,Hq,S] fp32 each, between the kernels of one call, and their work-queue counters: memory that
 * grows with S, not S^2, which is what the fused kernel is in the method for (Sec. 3.2; Sec. 2.4 "SP-3").  Returns 0
 * for an invalid shape.  Pure host arithmetic; touches no device.
 */
size_t ie_attn_bwd_workspace_bytes(int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D, int32_t num_docs);

/*
 * Bytes of workspace of the OPTIONAL backward path that trades memory for matrix work (selected with IE_BWD_STORED_DS
 * in ie_attn_bwd_phases, never by the size of the workspace alone).  For dense input (num_docs == 0) with
 * D == 128 and S a multiple of 128 this is ie_attn_bwd_workspace_bytes(...) plus room for dS = P o (dP - delta) in
 * bf16: B * Hq * S * (S + 128) bytes when causal (the lower block triangle of every head), 2 * B * Hq * S * S otherwise
 * (34.5 GB at B=1, S=32768, Hq=32).
 * On that path the dK/dV kernel stores the dS it forms and dQ = scale * dS K is computed from it, instead of
 * recomputing S, P and dP a second time for dQ (five matrix products per block pair instead of seven; the appendix "Implementation Detail: Selective Overlap" counts
 * the backward pass as the compute-heavier direction).  The results differ from the recomputing path only in
 * summation order (same bf16 dS, fp32 accumulation).  For every other shape the function returns
 * ie_attn_bwd_workspace_bytes(...): there is no such path.  Pure host arithmetic.
 */
size_t ie_attn_bwd_fast_workspace_bytes(int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D, int32_t num_docs,
                                        int32_t causal);

/*
 * Backward: given dout and the forward's o and lse, writes dq, dk, dv (fully
 * overwritten; dk/dv are summed over the Hq/Hkv query heads of each kv head).  The
 * probabilities are recomputed from lse (Sec. 3.2), backward costs 2.5x the forward's
 * matrix work (cf. the appendix "Implementation Detail: Selective Overlap": backward is about twice as compute-intensive as forward).
 * `workspace` is caller-owned scratch of at least ie_attn_bwd_workspace_bytes(...) bytes,
 * 256-byte aligned; its contents after the call are unspecified; a larger workspace changes nothing.  Every output element
 * has a single owner and a fixed summation order, so results are bitwise reproducible.
 */
int ie_attn_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout,
                const float* lse, void* dq, void* dk, void* dv,
                const int32_t* cu_seqlens, int32_t num_docs,
                int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D,
                float scale, int32_t causal,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same backward pass, restricted to some of its kernels, for profilers and benchmarks
 * that time one kernel at a time.  `phases` is a bit mask: IE_BWD_DELTA (delta = rowsum(dO o O)
 * and lse * log2(e), both negated, into the workspace), IE_BWD_DQ (writes dq; needs what IE_BWD_DELTA left in the
 * workspace), IE_BWD_DKDV (writes dk and dv; needs the same).  Outputs of phases that are not selected are left
 * untouched.  ie_attn_bwd(...) is ie_attn_bwd_phases(..., IE_BWD_ALL).
 * IE_BWD_STORED_DS, or-ed into the mask, selects the dS-storing path: the workspace must then have
 * ie_attn_bwd_fast_workspace_bytes(...) bytes (IE_ERR_WORKSPACE otherwise) and the shape must have that path
 * (IE_ERR_UNSUPPORTED otherwise).  There IE_BWD_DKDV also leaves dS in the workspace and IE_BWD_DQ needs it: run
 * IE_BWD_DKDV before IE_BWD_DQ.  A mask without a phase bit or with other bits set is IE_ERR_UNSUPPORTED.
 */
enum { IE_BWD_DELTA = 1, IE_BWD_DQ = 2, IE_BWD_DKDV = 4, IE_BWD_ALL = 7, IE_BWD_STORED_DS = 16 };
int ie_attn_bwd_phases(const void* q, const void* k, const void* v, const void* o, const void* dout,
                       const float* lse, void* dq, void* dk, void* dv,
                       const int32_t* cu_seqlens, int32_t num_docs,
                       int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D,
                       float scale, int32_t causal,
                       void* workspace, size_t workspace_bytes, int32_t phases, void* stream);

/*
 * The same forward and backward passes with q, k, v read where the first sequence-parallel all-to-all left them,
 * and dq, dk, dv written where the returning all-to-all picks them up: the re-layouts ie_sp_unpack_qkv and
 * ie_sp_pack_dqkv (ie_sp.h) disappear from the layer (Sec. 2.4 "SP-2": after the exchange every GPU holds the
 * complete sequence of Q, K, V for its heads; Sec. 3.2.2: the same exchanges run in the backward pass).
 * `xqkv` is the received exchange buffer of ie_sp.h, [P][B][ q:[Sl][Hq/P][D] | k:[Sl][Hkv/P][D] | v:[Sl][Hkv/P][D] ]
 * (chunk p = tokens [p*Sl, (p+1)*Sl) of this GPU's heads), `dxqkv` a buffer of the same layout that receives
 * dq | dk | dv.  o, dout [B][P*Sl][Hq/P][D] and lse [B][Hq/P][P*Sl] are as in ie_attn_fwd / ie_attn_bwd (with B == 1
 * that IS the layout the second exchange sends and receives).  Hq, Hkv are the head counts of the whole layer, both
 * divisible by P; Sl must be a power of two and at least 256 (IE_ERR_UNSUPPORTED otherwise: use the re-layouts);
 * dense input only.  The workspace is that of ie_attn_bwd for (B, P*Sl, Hq/P, Hkv/P, D).  Results are bit-identical
 * to unpacking, calling ie_attn_fwd / ie_attn_bwd and packing.
 */
int ie_attn_fwd_sp(const void* xqkv, void* o, float* lse,
                   int64_t B, int64_t Sl, int32_t Hq, int32_t Hkv, int32_t D, int32_t P,
                   float scale, int32_t causal, void* stream);
int ie_attn_bwd_sp(const void* xqkv, const void* o, const void* dout, const float* lse, void* dxqkv,
                   int64_t B, int64_t Sl, int32_t Hq, int32_t Hkv, int32_t D, int32_t P,
                   float scale, int32_t causal,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * ie_attn_bwd for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The same computation and the same kernels as ie_attn_bwd(...) with the minimal
 * workspace, but the workspace is a device array inside the library (IE_ATTN_BWD_STATIC_MAX_ROWS * 8 + 256 bytes,
 * about 16 MiB, held on every device the library runs on until the process ends), so the call takes no workspace
 * argument and neither it nor anything it calls allocates or frees memory.  Shapes with
 * B * Hq * S > IE_ATTN_BWD_STATIC_MAX_ROWS are rejected with IE_ERR_WORKSPACE before anything is launched.  All
 * calls on one device share the array: calls that overlap on one device (different streams, or two replays of a
 * captured graph at once) race and give undefined results; calls on one stream are safe.  Results are bit-identical
 * to ie_attn_bwd's.
 */
#define IE_ATTN_BWD_STATIC_MAX_ROWS (1 << 21)
int ie_attn_bwd_static(const void* q, const void* k, const void* v, const void* o, const void* dout,
                       const float* lse, void* dq, void* dk, void* dv,
                       const int32_t* cu_seqlens, int32_t num_docs,
                       int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D,
                       float scale, int32_t causal, void* stream);

/*
 * Query rows per work item at head dimension 128, for the forward and the recomputing dQ kernel: 256
 * (one persistent workgroup per CU; the faster steady state) or 128 (two workgroups per CU; half the
 * work per item, which wins when a launch has few items per CU or the sequence is short).  rows = 0
 * (the initial setting) lets every call choose from its shape: dense input of up to 4096 tokens, or
 * up to 8192 tokens with fewer than two 256-row items per CU, takes the 128-row forward; dense input
 * of 8192 tokens or more with fewer than two 256-row items per CU takes the 128-row dQ.  rows = 128
 * or 256 fixes the choice for all later calls of the process (measurements, tests); the results of
 * the two differ only in rounding order.  Returns the previous setting, or IE_ERR_UNSUPPORTED for any
 * other value.  Head dimension 64 always works on 128-row items.  (Sec. 4.2: self-atten is profiled
 * over shapes from 4K x 40 heads to 256K x 1 head per GPU.)
 */
int ie_attn_set_tile_rows(int32_t rows);

/* Static text for a status code (never NULL). */
const char* ie_attn_strerror(int code);

/* Text of the HIP error behind the calling thread's most recent IE_ERR_HIP ("" if none). */
const char* ie_attn_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* IE_ATTN_H */
