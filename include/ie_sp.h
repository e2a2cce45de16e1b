/*
 * ie_sp — the local re-layouts either side of the sequence-parallel all-to-all (MI355X / gfx950).
 *
 * With sequence parallelism of degree P = s_sp and no tensor parallelism, every module except
 * attention works on a slice of S/P tokens with all heads, and attention works on all S tokens
 * with heads/P heads; an all-to-all before attention and one after it change between the two
 * partitions (Sec. 2.4 "SP-2"; Sec. 3.2.2 "Sequence Parallelism": 6bSH bytes in the first
 * exchange, 2bSH in the second, per layer and direction).  An all-to-all moves P equal,
 * contiguous chunks, chunk p to and from peer p; the tensors on either side are not laid out that
 * way, so each exchange has a local permutation before it ("pack") and one after it ("unpack").
 * These eight functions are those permutations, for the forward pass (qkv before attention, o after
 * it) and for the backward pass (dout before, dq/dk/dv after).  They move bf16 values as
 * 16-bit patterns: outputs are bit-exact copies.  The exchange itself is not part of this library.
 *
 * Notation: P peers; Sl = S/P tokens per sequence slice; Hq, Hkv = heads of the whole layer
 * (both divisible by P); Hql = Hq/P, Hkvl = Hkv/P heads per peer; head group p = heads
 * [p*Hl, (p+1)*Hl); sequence slice p = tokens [p*Sl, (p+1)*Sl).
 *
 * Layouts (all contiguous, bf16; "|" is concatenation):
 *   qkv_local  [B][ q:[Sl][Hq][D] | k:[Sl][Hkv][D] | v:[Sl][Hkv][D] ]
 *              the fused QKV projection of this GPU's sequence slice; with Hq == Hkv this is the
 *              B x 3 x S/s_sp x H tensor of Sec. 2.4.
 *   xqkv       [P][B][ q:[Sl][Hql][D] | k:[Sl][Hkvl][D] | v:[Sl][Hkvl][D] ]
 *              exchange buffer of the first all-to-all.  Sent: chunk p = head group p of this
 *              GPU's sequence slice.  Received: chunk p = sequence slice p of this GPU's head group.
 *   q, o, dout, dq   [B][P*Sl][Hql][D]   and   k, v, dk, dv   [B][P*Sl][Hkvl][D]
 *              the attention kernels' operands (ie_attn.h) for this GPU's head group.
 *   xo         [P][B][Sl][Hql][D]
 *              exchange buffer of the second all-to-all.  Sent: chunk p = sequence slice p of this
 *              GPU's head group.  Received: chunk p = head group p of this GPU's sequence slice.
 *   o_local, dout_local   [B][Sl][Hq][D]
 *              attention output (gradient) of this GPU's sequence slice, all heads.
 *
 * Conventions: as in ie_attn.h (device pointers owned by the caller, work enqueued on `stream`,
 * no host synchronisation, no allocation, status codes of ie_attn_status).  Source and destination
 * must not overlap.  Every pointer must be 16-byte aligned (IE_ERR_ALIGN).  Supported: P, B, Sl,
 * Hq, Hkv >= 1 with Hq % P == 0 and Hkv % P == 0, P * B <= 65535 and every buffer below 2^40 elements
 * (IE_ERR_SHAPE otherwise), D a positive multiple of 8 (IE_ERR_UNSUPPORTED otherwise).  Outputs are
 * fully overwritten.  On error nothing has been launched, except for IE_ERR_HIP.
 * With B == 1 the layouts of o (dout) and xo coincide (the sequence slices of [1][P*Sl][Hql][D] are already
 * contiguous chunks): ie_sp_pack_o and ie_sp_unpack_do are then plain copies, and a caller may hand o
 * to the exchange directly and receive dout in place.
 */
#ifndef IE_SP_H
#define IE_SP_H

#include "ie_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Forward, before the first all-to-all (Sec. 2.4 "SP-2": the output of Linear_qkv is exchanged):
 * xqkv[p][b][t][s][hl][:] = qkv_local[b][t][s][p*Hl_t + hl][:], t in {q, k, v}. */
int ie_sp_pack_qkv(const void* qkv_local, void* xqkv, int64_t B, int64_t Sl, int32_t Hq, int32_t Hkv, int32_t D,
                   int32_t P, void* stream);

/* Forward, after the first all-to-all (Sec. 2.4: every GPU then holds the complete sequence of Q, K
 * and V for a subset of the heads): t[b][p*Sl + s][hl][:] = xqkv[p][b][t][s][hl][:]. */
int ie_sp_unpack_qkv(const void* xqkv, void* q, void* k, void* v, int64_t B, int64_t Sl, int32_t Hq, int32_t Hkv,
                     int32_t D, int32_t P, void* stream);

/* Forward, before the second all-to-all (Sec. 2.4: the attention results are gathered and
 * re-partitioned along the sequence): xo[p][b][s][hl][:] = o[b][p*Sl + s][hl][:]. */
int ie_sp_pack_o(const void* o, void* xo, int64_t B, int64_t Sl, int32_t Hq, int32_t D, int32_t P, void* stream);

/* Forward, after the second all-to-all: o_local[b][s][p*Hql + hl][:] = xo[p][b][s][hl][:]. */
int ie_sp_unpack_o(const void* xo, void* o_local, int64_t B, int64_t Sl, int32_t Hq, int32_t D, int32_t P,
                   void* stream);

/* Backward (Sec. 3.2.2: the same two exchanges run in the backward pass).  Each is the inverse
 * permutation of a forward function, applied to the gradient that flows the other way:
 *   ie_sp_pack_do     inverts ie_sp_unpack_o :  xo[p][b][s][hl][:]  = dout_local[b][s][p*Hql + hl][:]
 *   ie_sp_unpack_do   inverts ie_sp_pack_o   :  dout[b][p*Sl + s][hl][:] = xo[p][b][s][hl][:]
 *   ie_sp_pack_dqkv   inverts ie_sp_unpack_qkv: xqkv[p][b][t][s][hl][:] = dt[b][p*Sl + s][hl][:]
 *   ie_sp_unpack_dqkv inverts ie_sp_pack_qkv :  dqkv_local[b][t][s][p*Hl_t + hl][:] = xqkv[p][b][t][s][hl][:]
 */
int ie_sp_pack_do(const void* dout_local, void* xo, int64_t B, int64_t Sl, int32_t Hq, int32_t D, int32_t P,
                  void* stream);
int ie_sp_unpack_do(const void* xo, void* dout, int64_t B, int64_t Sl, int32_t Hq, int32_t D, int32_t P,
                    void* stream);
int ie_sp_pack_dqkv(const void* dq, const void* dk, const void* dv, void* xqkv, int64_t B, int64_t Sl, int32_t Hq,
                    int32_t Hkv, int32_t D, int32_t P, void* stream);
int ie_sp_unpack_dqkv(const void* xqkv, void* dqkv_local, int64_t B, int64_t Sl, int32_t Hq, int32_t Hkv, int32_t D,
                      int32_t P, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* IE_SP_H */
