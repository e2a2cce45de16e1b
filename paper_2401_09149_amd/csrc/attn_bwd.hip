// Backward kernels.  The probabilities are recomputed from the saved log-sum-exp (the
// fused kernel's selective recomputation, Sec. 3.2), and the five products of the
// backward pass (the appendix "Implementation Detail: Selective Overlap": backward is the compute-heavier direction) are split over two
// kernels so that each output has exactly one owner and nothing is accumulated through
// memory:
//   attn_bwd_delta : delta_i = <dO_i, O_i>                              (HBM-bound)
//   attn_bwd_dq    : query-stationary, like the forward: S^T = K Q^T, dP^T = V dO^T,
//                    dS^T = P^T o (dP^T - delta), dQ^T += K^T dS^T
//   attn_bwd_dkdv  : key-stationary: S = Q K^T, dP = dO V^T, dV^T += dO^T P,
//                    dK^T += Q^T dS, looping over the query heads of the kv head's group
// When the caller's workspace has room for it, the dK/dV kernel also stores dS and dQ comes from
//   attn_bwd_dq_from_ds : dQ^T += K^T dS^T, a stream over the stored dS (five products in all instead of seven)
// In both main kernels the elementwise results leave the first products in the C layout
// (one column per lane, rows over registers) with the NEXT contraction index on the
// rows, so they feed the following MFMA from registers; the transposed operands
// (K^T, dO^T, Q^T) are gathered from row-major LDS tiles with transpose loads.
#include <type_traits>

#include "attn_common.hpp"
#include "launch.hpp"
#include "mfma_asm.hpp"
#include "tile_queue.hpp"

namespace ie {

// ---- delta = rowsum(dO o O) ------------------------------------------------------------
// HBM-bound: o and dO are read once, 2 * T * Hq * D * 2 bytes.  A workgroup takes kDeltaTokens consecutive
// tokens of one batch entry with ALL their heads, which is one contiguous piece of o and of dO (the layout is
// [B, S, Hq, D]), and walks it front to back with D/8 lanes per (token, head) row and eight rows per thread in
// flight.  The sums are parked in LDS as [head][token] and written out from there, so that the [B, Hq, S]
// planes receive runs of kDeltaTokens consecutive floats.  The same pass stores lse * log2(e) next to delta.
// Both are stored NEGATED: -delta is the C operand of the first MFMA of every dP chain, which then delivers
// dP - delta directly, and -lse*log2(e) is the addend of the fused multiply-add in front of each exp2.
constexpr int kDeltaTokens = 32;   // per workgroup; fewer (p.tiles) when Hq * 32 floats would not fit the default LDS limit
template <int D>
__global__ __launch_bounds__(kThreads) void attn_bwd_delta_kernel(AttnParams p) {
  constexpr int LPR = D / 8;               // lanes per row
  constexpr int RPP = kThreads / LPR;      // rows per pass of the workgroup
  constexpr int UNROLL = 8;
  extern __shared__ float s_delta[];       // [Hq][tokens per workgroup]
  const int kTok = p.tiles;                // tokens per workgroup
  const int tid = threadIdx.x;
  // The work-queue counters of the two kernels that follow on this stream (tile_queue.hpp) are cleared here, which
  // saves each of them a launch of its own in front.
  if (blockIdx.x == 0 && tid < 2 * (kQueueBytes / 4)) p.ws_counters[tid] = 0u;
  const int sub = tid % LPR, rloc = tid / LPR;
  const int64_t blocks_per_batch = (p.S + kTok - 1) / kTok;
  const int64_t b = blockIdx.x / blocks_per_batch;
  const int64_t t0 = (blockIdx.x % blocks_per_batch) * kTok;
  const int ntok = (int)(p.S - t0 < kTok ? p.S - t0 : kTok);
  const int rows = ntok * p.Hq;            // (token, head) rows of this workgroup, contiguous in memory
  const __bf16* o = p.o + (b * p.S + t0) * p.Hq * D;
  const __bf16* dout = p.dout + (b * p.S + t0) * p.Hq * D;
  for (int r0 = 0; r0 < rows; r0 += RPP * UNROLL) {
    bf16x8 x[UNROLL], y[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int r = r0 + u * RPP + rloc;
      const int rr = r < rows ? r : rows - 1;   // clamped copies are computed and dropped
      x[u] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(o + (int64_t)rr * D + sub * 8));
      y[u] = *reinterpret_cast<const bf16x8*>(dout + (int64_t)rr * D + sub * 8);
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      float acc = 0.f;
#pragma unroll
      for (int t = 0; t < 8; ++t) acc = __builtin_fmaf((float)x[u][t], (float)y[u][t], acc);
#pragma unroll
      for (int s = LPR / 2; s >= 1; s >>= 1) acc += __shfl_xor(acc, s, 64);
      const int r = r0 + u * RPP + rloc;
      if (sub == 0 && r < rows) s_delta[(r % p.Hq) * kTok + r / p.Hq] = -acc;
    }
  }
  __syncthreads();
  for (int idx = tid; idx < p.Hq * kTok; idx += kThreads) {
    const int h = idx / kTok, t = idx % kTok;
    if (t < ntok) {
      const int64_t at = (b * p.Hq + h) * p.S + t0 + t;
      p.delta[at] = s_delta[idx];
      p.lse2[at] = -p.lse[at] * kLog2e;
    }
  }
}

// ---- dQ ----------------------------------------------------------------------------------
// Same skeleton as the narrow forward kernel: 32 query rows per wave (Q and dO fragments in registers), 64-key K/V
// tiles double-buffered in LDS by asynchronous copies, each consumed as two 32-key blocks.  WAVES = 4: 128 query rows
// per workgroup, two workgroups per CU.  WAVES = 8: 256 query rows per workgroup, one workgroup per CU with two waves
// per SIMD, so that every K/V tile is copied into LDS once per 256 queries instead of once per 128.
template <int WAVES>
struct DqCfg {
  static constexpr int THREADS = 64 * WAVES;
  static constexpr int BM = 32 * WAVES;
  static constexpr int BN = 64;   // keys per LDS stage (128-key stages were 2 % slower with either workgroup size)
  template <int D> static constexpr int smem_bytes() { return 2 * 2 * BN * D * 2; }   // two stages of a K and a V tile
};
template <int D, int WAVES>
__global__ __launch_bounds__(64 * WAVES, 8 / WAVES) void attn_bwd_dq_kernel(AttnParams p) {
  constexpr int BM = DqCfg<WAVES>::BM, BN = DqCfg<WAVES>::BN, THREADS = DqCfg<WAVES>::THREADS;
  constexpr int NKS = D / 16, NDB = D / 32;
  constexpr int TILE_BYTES = BN * D * 2;
  constexpr int STAGE_BYTES = 2 * TILE_BYTES;
  constexpr int ROW_BYTES = D * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ int scratch[2 * WAVES + 2];

  __shared__ QueueState s_work;
  queue_init(p, &s_work);
  const uint32_t xcc = xcc_id();
  int skip = 0;
  for (;;) {   // persistent: one item (batch, head, query tile) per iteration (tile_queue.hpp)
  const int item = next_work(p, &s_work, xcc, skip);
  if (item < 0) break;
  // (an opaque copy of the thread index: per-lane offsets are recomputed per item rather than
  // hoisted out of this loop and kept in registers through the main loop)
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wv = tid >> 6;
  const int n = lane & 31, h = lane >> 5, grp = lane >> 4;

  TileCoord tc = decode_tile<BM, THREADS>(p, p.Hq, true, scratch, item, tid);
  if (!tc.valid) continue;
  // (the tile coordinates may have come through LDS: wave-uniform values are moved to scalar registers explicitly)
  const int g = tc.h / (p.Hq / p.Hkv);
  const int64_t q0 = uniform(tc.t0), doc_end = uniform(tc.doc_end);
  const int64_t q_end = (q0 + BM < doc_end) ? q0 + BM : doc_end;
  const int64_t k_begin = uniform(tc.doc_begin);
  const int64_t k_end = p.causal ? q_end : doc_end;
  const int nk = (int)(k_end - k_begin);
  const int nkt = (nk + BN - 1) / BN;
  const int nfull = nk / BN;

  const int64_t q_stride = (int64_t)p.Hq * D;
  const int64_t kv_pitch = (int64_t)p.Hkv * D * 2;
  const int64_t qhead = ((int64_t)tc.b * p.S * p.Hq + tc.h) * D;   // for dout (always contiguous)
  const char* kbase = uniform(reinterpret_cast<const char*>(p.k + g * D) + tc.b * p.kv_bstride);   // key tile kt starts at token k_begin + kt * BN
  const char* vbase = uniform(reinterpret_cast<const char*>(p.v + g * D) + tc.b * p.kv_bstride);
  auto key_tile_off = [&](const int kt) __attribute__((always_inline)) { return tok_off(p, k_begin + (int64_t)kt * BN, kv_pitch); };

  const uint32_t lds0 = lds_address(smem);
  AsyncTile<D, WAVES> ld;
  ld.init(tid, kv_pitch);
  // Asynchronous copy of key tile kt, of which `rows` >= 1 rows exist, into the stage at LDS address `lds`, in
  // 64-row parts; a part that lies past the end repeats the last valid row (masked later).
  auto load_kv = [&](const uint32_t lds, const int kt, const int rows, auto full) __attribute__((always_inline)) {
    const int64_t off = key_tile_off(kt);
#pragma unroll
    for (int part = 0; part < BN / 64; ++part) {
      const uint32_t dst = lds + part * 64 * ROW_BYTES;
      if (full) {
        ld.load_full(dst, kbase + off + (int64_t)(64 * part) * kv_pitch);
        ld.load_full(dst + TILE_BYTES, vbase + off + (int64_t)(64 * part) * kv_pitch);
      } else {
        const int first = rows > 64 * part ? 64 * part : rows - 1;
        const int valid = rows > 64 * part ? rows - 64 * part : 1;
        ld.load(dst, kbase + off + (int64_t)first * kv_pitch, valid);
        ld.load(dst + TILE_BYTES, vbase + off + (int64_t)first * kv_pitch, valid);
      }
    }
  };
  load_kv(lds0, 0, nk, std::false_type{});

  // This lane's query row, as a 32-bit position inside the document (rows past the tile's end repeat its last row and
  // are not written).
  const int rows_rel_end = (int)(q_end - k_begin);
  const int row_rel_raw = (int)(q0 - k_begin) + wv * 32 + n;
  const int row_rel = row_rel_raw < rows_rel_end ? row_rel_raw : rows_rel_end - 1;
  const int64_t row = k_begin + row_rel;

  bf16x8 qf[NKS], dof[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    qf[ks] = *reinterpret_cast<const bf16x8*>(reinterpret_cast<const char*>(p.q + tc.h * D) + tc.b * p.q_bstride +
                                              tok_off(p, row, q_stride * 2) + (ks * 16 + h * 8) * 2);
    dof[ks] = *reinterpret_cast<const bf16x8*>(p.dout + qhead + row * q_stride + ks * 16 + h * 8);
  }
  const int64_t stat = ((int64_t)tc.b * p.Hq + tc.h) * p.S + row;
  const float nlse2 = p.lse2[stat];    // -lse * log2(e) of this lane's query
  const float ndelta = p.delta[stat];  // -delta

  const char* nat_ptr[NKS];  // row n of a tile, chunk 2ks + h (A operand: K or V rows)
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) nat_ptr[ks] = smem + tile_off<D>(n, 2 * ks + h);
  const char* tr_ptr0[NDB];  // transpose loads on the K tile
  const char* tr_ptr8[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    tr_ptr0[db] = smem + tr_off<D>(lane, 4 * (grp >> 1), 32 * db + 16 * (grp & 1));
    tr_ptr8[db] = smem + tr_off<D>(lane, 8 + 4 * (grp >> 1), 32 * db + 16 * (grp & 1));
  }

  // The dP chain starts from -delta (the same value in all 16 rows: one query per lane), so it
  // delivers dP - delta.
  const float c = p.scale_log2;
  f32x16 dp_init;
#pragma unroll
  for (int r = 0; r < 16; ++r) dp_init[r] = ndelta;
  f32x16 acc[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

  const int wave_row_min = (int)(q0 - k_begin) + wv * 32;

  auto tile_step = [&](const int kt, const int stage, auto full_next) __attribute__((always_inline)) {
    const int kb = kt * BN;
    const uint32_t next_lds = lds0 + (STAGE_BYTES - stage);
    if (full_next) load_kv(next_lds, kt + 1, BN, std::true_type{});
    else if (kt + 1 < nkt) load_kv(next_lds, kt + 1, nk - kb - BN, std::false_type{});
    const bool need_mask = (p.causal && kb + BN - 1 > wave_row_min) || (kb + BN > nk);
    const int lim = (p.causal ? row_rel : nk - 1) - kb - 4 * h;

#pragma unroll
    for (int j = 0; j < BN / 32; ++j) {
      const int blk = stage + 32 * j * ROW_BYTES;
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) s = mfma32(lds_read8(nat_ptr[ks], blk), qf[ks], s);
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) dp = mfma32(lds_read8(nat_ptr[ks], blk + TILE_BYTES), dof[ks], ks == 0 ? dp_init : dp);
      // K^T fragments for the dQ product: the first 16 keys' are requested before the
      // elementwise work, the other 16 keys' while the first half of dS is being formed
      bf16x8 ktf[2][NDB];
      auto load_ktf = [&](int sblk) __attribute__((always_inline)) {
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          const int off = blk + 16 * sblk * ROW_BYTES;
          ktf[sblk][db] = cat4(lds_read_tr4(tr_ptr0[db] + off), lds_read_tr4(tr_ptr8[db] + off));
        }
      };
      load_ktf(0);
      if (need_mask) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (32 * j + 8 * (r >> 2) + (r & 3) > lim) s[r] = -INFINITY;
      }
      bf16x8 dsf[2];
#pragma unroll
      for (int sblk = 0; sblk < 2; ++sblk) {
        if (sblk == 1) load_ktf(1);
        bf16x2 pr[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int r = 8 * sblk + 2 * t;
          const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, nlse2));
          const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r + 1], c, nlse2));
          pr[t] = pack_bf16(p0 * dp[r], p1 * dp[r + 1]);
        }
        dsf[sblk] = cat_pairs(pr[0], pr[1], pr[2], pr[3]);
      }
      // dQ^T += K^T dS^T over this block's 32 keys
#pragma unroll
      for (int sblk = 0; sblk < 2; ++sblk)
#pragma unroll
        for (int db = 0; db < NDB; ++db) acc[db] = mfma32(ktf[sblk][db], dsf[sblk], acc[db]);
    }
    async_wait_all();
    __syncthreads();
  };

#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) { consume(qf[ks]); consume(dof[ks]); }
  consume(nlse2);
  consume(ndelta);
  async_wait_all();
  __syncthreads();
  int kt = 0;
  for (; kt + 2 < nfull; kt += 2) {
    tile_step(kt, 0, std::true_type{});
    tile_step(kt + 1, STAGE_BYTES, std::true_type{});
  }
  for (; kt < nkt; ++kt) tile_step(kt, (kt & 1) * STAGE_BYTES, std::false_type{});

  // (the row is formed again from its 32-bit position: a 64-bit row index kept alive through the main loop is two
  // registers this kernel does not have)
  int row_rel_late = row_rel;
  asm volatile("" : "+v"(row_rel_late));   // (opaque: otherwise the address is formed in the prologue all the same)
  __bf16* drow = reinterpret_cast<__bf16*>(reinterpret_cast<char*>(p.dq + tc.h * D) + tc.b * p.q_bstride +
                                           tok_off(p, k_begin + row_rel_late, q_stride * 2));
#pragma unroll
  for (int db = 0; db < NDB; ++db) store_block32_bf16(drow + 32 * db, acc[db], p.scale, h, wave_row_min + n < rows_rel_end);
  }  // next item
}

// ---- dK, dV ------------------------------------------------------------------------------
// One workgroup per (batch, kv head, 128 keys); wave w owns keys 32w..32w+31 and keeps their
// K and V fragments and the dK^T / dV^T accumulators in registers for the whole kernel.
// Query tiles of 128 rows (Q, dO, -lse*log2e, -delta) stream through two LDS stages
// filled by asynchronous copies; all query heads of the kv head's group pass through the
// same accumulators, which is the GQA reduction.
template <int D>
struct DkdvCfg {
  static constexpr int BK = 128;                                  // keys per workgroup
  static constexpr int BQ = 128;                                  // query rows per loop step
  static constexpr int NB = BQ / 32;                              // 32-row blocks per step
  static constexpr int TILE_BYTES = BQ * D * 2;
  static constexpr int STAT_BYTES = 2 * BQ * 4;                   // lse*log2e [BQ], delta [BQ]
  static constexpr int STAGE_BYTES = 2 * TILE_BYTES + STAT_BYTES; // Q, dO, stats
  static constexpr int STAGES = 2;
  static constexpr int SMEM_BYTES = STAGES * STAGE_BYTES;
};

// CHUNKED: q, k, v, dk, dv are chunks of a sequence-parallel exchange buffer (tok_off in attn_common.hpp) instead of
// contiguous tensors: a separate instantiation, so that the contiguous case keeps its simpler address arithmetic.
template <int D, bool STORE_DS, bool CHUNKED = false>
__global__ __launch_bounds__(kThreads, 1) void attn_bwd_dkdv_kernel(AttnParams p) {
  static_assert(!(STORE_DS && CHUNKED), "the stored-dS path takes contiguous tensors");
  using C = DkdvCfg<D>;
  constexpr int BK = C::BK, BQ = C::BQ, NB = C::NB;
  constexpr int NKS = D / 16, NDB = D / 32;
  constexpr int TILE_BYTES = C::TILE_BYTES, STAGE_BYTES = C::STAGE_BYTES;
  constexpr int ROW_BYTES = D * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ int scratch[8];

  __shared__ QueueState s_work;
  queue_init(p, &s_work);
  const uint32_t xcc = xcc_id();
  int skip = 0;
  for (;;) {   // persistent: one item (batch, kv head, key block) per iteration (tile_queue.hpp)
  const int item = next_work(p, &s_work, xcc, skip);
  if (item < 0) break;
  // (an opaque copy of the thread index: per-lane offsets are recomputed per item rather than
  // hoisted out of this loop and kept in registers through the main loop)
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wv = tid >> 6;
  const int n = lane & 31, h = lane >> 5, grp = lane >> 4;

  TileCoord tc = decode_tile<BK>(p, p.Hkv, false, scratch, item, tid);
  if (!tc.valid) continue;
  // The tile coordinates may have come through LDS (packed input): they are the same in every lane, and are moved
  // to scalar registers here so that everything derived from them between two steps (the description of the next
  // query tile: three 64-bit addresses) is scalar arithmetic instead of vector multiplies and lane reads.
  tc.b = (int)uniform((uint32_t)tc.b);
  tc.h = (int)uniform((uint32_t)tc.h);
  tc.t0 = uniform(tc.t0);
  tc.doc_begin = uniform(tc.doc_begin);
  tc.doc_end = uniform(tc.doc_end);
  const int g = tc.h;
  const int group = (int)uniform((uint32_t)(p.Hq / p.Hkv));   // (an integer division leaves its result in a vector register)
  const int64_t k0 = tc.t0;
  const int64_t q_begin = p.causal ? k0 : tc.doc_begin;
  const int nq = (int)(tc.doc_end - q_begin);  // query rows that can see this key tile
  const int nqt = (nq + BQ - 1) / BQ;
  const int total = nqt * group;               // loop steps: query heads of the group x query tiles

  const int64_t q_pitch = (int64_t)p.Hq * D * 2;  // bytes between consecutive tokens of one query head
  const int64_t kv_pitch = (int64_t)p.Hkv * D * 2;   // bytes between consecutive tokens of one kv head
  // bytes: head g of the batch entry's first token
  const int64_t kvhead = CHUNKED ? tc.b * p.kv_bstride + (int64_t)g * D * 2 : ((int64_t)tc.b * p.S * p.Hkv + g) * D * 2;
  auto kv_row_off = [&](const int64_t t) __attribute__((always_inline)) {
    if constexpr (CHUNKED) return tok_off(p, t, kv_pitch);
    else return t * kv_pitch;
  };

  const uint32_t lds0 = lds_address(smem);
  AsyncTile<D> ld;
  ld.init(tid, q_pitch);
  const int wave_u = ld.wave;

  // Asynchronous copy of one (query head, query tile) into a stage.  The tile is described once
  // (scalar arithmetic only) and then copied either all at once or piece by piece: a wave issues
  // in order, and 17 back-to-back copy instructions hold it for as long as the memory pipeline
  // needs to accept them (about 1 KiB per 16 cycles per CU), so the hand-sequenced tile spreads
  // them between its MFMA chains.
  struct TileCopy {
    const char* qg;    // first row of the Q tile of that head
    const char* dog;   // first row of the dO tile
    const char* stat;  // lse*log2e (waves 0,1) or delta (waves 2,3) of the tile's first row
    int rows;          // valid rows, >= 1
    uint32_t base;     // LDS address of the stage
  };
  constexpr int kPieces = 2 * (BQ / 64) * AsyncTile<D>::NI + 1;
  auto describe = [&](const int hq_idx, const int tile_idx, const int slot) __attribute__((always_inline)) {
    TileCopy t;
    const int hq = g * group + hq_idx;
    const int i0 = tile_idx * BQ;  // first row of the tile, relative to q_begin
    t.rows = nq - i0;
    const int64_t tok = (int64_t)tc.b * p.S + q_begin + i0;
    if constexpr (CHUNKED) t.qg = reinterpret_cast<const char*>(p.q + hq * D) + tc.b * p.q_bstride + tok_off(p, q_begin + i0, q_pitch);
    else t.qg = reinterpret_cast<const char*>(p.q + (tok * p.Hq + hq) * D);
    t.dog = reinterpret_cast<const char*>(p.dout + (tok * p.Hq + hq) * D);
    const int64_t idx = ((int64_t)tc.b * p.Hq + hq) * p.S + q_begin + i0;
    t.stat = reinterpret_cast<const char*>((wave_u < 2 ? p.lse2 : p.delta) + idx);
    t.base = lds0 + slot * STAGE_BYTES;
    return t;
  };
  // statistics, one dword per lane = one row: waves 0,1 copy lse*log2e of rows 0-63, 64-127;
  // waves 2,3 copy delta.  Rows past the end repeat the last valid row (masked later).
  auto copy_stats = [&](const TileCopy& t) __attribute__((always_inline)) {
    const int half = wave_u & 1;
    int r = 64 * half + lane;
    r = r < t.rows ? r : t.rows - 1;
    const char* src = uniform(t.stat);
    const uint32_t dst = uniform(t.base + 2 * TILE_BYTES + (wave_u < 2 ? 0 : BQ * 4) + half * 256);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :
                 : "v"((uint32_t)r * 4u), "s"(src), "s"(dst)
                 : "memory");
  };
  auto copy_all = [&](const TileCopy& t) __attribute__((always_inline)) {
#pragma unroll
    for (int part = 0; part < BQ / 64; ++part) {
      // a part that lies entirely past the end repeats the last valid row 64 times
      const int first = t.rows > 64 * part ? 64 * part : t.rows - 1;
      const int valid = t.rows > 64 * part ? t.rows - 64 * part : 1;
      ld.load(t.base + part * 64 * ROW_BYTES, t.qg + (int64_t)first * q_pitch, valid);
      ld.load(t.base + TILE_BYTES + part * 64 * ROW_BYTES, t.dog + (int64_t)first * q_pitch, valid);
    }
    copy_stats(t);
  };
  // piece k of a tile that is known to have all BQ rows
  auto copy_piece = [&](const TileCopy& t, const int k) __attribute__((always_inline)) {
    constexpr int NI = AsyncTile<D>::NI, RPI = AsyncTile<D>::RPI;
    if (k == kPieces - 1) {
      copy_stats(t);
    } else {
      const int tensor = k / ((BQ / 64) * NI), part = (k / NI) % (BQ / 64), i = k % NI;
      const int row = 64 * part + 4 * RPI * i;
      async_copy16(ld.voff, (tensor ? t.dog : t.qg) + (int64_t)row * q_pitch,
                   t.base + tensor * TILE_BYTES + part * 64 * ROW_BYTES + (i * 4 + wave_u) * 1024);
    }
  };
  copy_all(describe(0, 0, 0));

  // This lane's key (column of S); clamped copies are computed but never written.
  int64_t key = k0 + wv * 32 + n;
  const bool key_ok = key < tc.doc_end;
  const int key_rel = (int)(key - q_begin);  // position of the key among the rows that see the tile
  // dS workspace (STORE_DS): this lane's 32-byte slot inside the block of the step's (query head, query
  // tile), for 32-query block 0 (block rb adds 2048); the block itself is located once per step (ds_step)
  const uint32_t ds_lane = (uint32_t)(k0 / 32 + wv) * 8192u + (uint32_t)h * 1024u + (uint32_t)((n ^ (h << 2)) << 5);
  // (dense input, S a multiple of 128: the step's query tile is it0 + tile_idx)
  const int it0 = (int)((q_begin - tc.doc_begin) / BQ);
  const int64_t ds_head = STORE_DS ? ds_matrix_offset(p.S / BQ, 1, 0, p.causal != 0) : 0;
  char* ds_first = STORE_DS ? reinterpret_cast<char*>(p.ds) + ds_matrix_offset(p.S / BQ, (int64_t)tc.b * p.Hq + g * group, it0, p.causal != 0)
                            : nullptr;   // first step of the current query head
  char* ds_step = ds_first;
  // The item's K and V rows reach their registers through the second LDS stage, which is free until the first step
  // copies the second query tile into it: two coalesced tile copies and one 16-byte LDS read per fragment.  (Loaded
  // straight from memory, a fragment instruction gathers 32 bytes from each of 32 rows: 2.7 us per item for the 16 of
  // them against 1 us for the copies.)  Keys past the document's end repeat its last key, as key_ld does.
  bf16x8 kf[NKS], vf[NKS];                   // live in AGPRs
  {
    AsyncTile<D> ldk;
    ldk.init(tid, kv_pitch);
    const int keys = (int)((tc.doc_end - k0 < BK) ? tc.doc_end - k0 : BK);   // >= 1
    const char* ksrc = reinterpret_cast<const char*>(p.k) + kvhead + kv_row_off(k0);
    const char* vsrc = reinterpret_cast<const char*>(p.v) + kvhead + kv_row_off(k0);
#pragma unroll
    for (int part = 0; part < BK / 64; ++part) {
      const int first = keys > 64 * part ? 64 * part : keys - 1;
      const int valid = keys > 64 * part ? keys - 64 * part : 1;
      ldk.load(lds0 + STAGE_BYTES + part * 64 * ROW_BYTES, ksrc + (int64_t)first * kv_pitch, valid);
      ldk.load(lds0 + STAGE_BYTES + TILE_BYTES + part * 64 * ROW_BYTES, vsrc + (int64_t)first * kv_pitch, valid);
    }
    async_wait_all();
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      const uint32_t a = lds0 + STAGE_BYTES + (uint32_t)(wv * 32 * ROW_BYTES) + (uint32_t)tile_off<D>(n, 2 * ks + h);
      kf[ks] = lds_load_to_agpr(a);
      vf[ks] = lds_load_to_agpr(a + TILE_BYTES);
    }
  }

  // Per-lane LDS addresses for each stage; block, tile and k-step offsets are immediates.
  struct StagePtrs {
    const char* nat[NKS];   // row n of a tile, chunk 2ks + h (A operand: Q or dO rows)
    const char* tr0[NDB];   // transpose loads, rows 4h.. of a 16-row group
    const char* tr8[NDB];   // rows 8 + 4h..
    const char* stat;       // this half-wave's 4-row groups of the statistics
  } sp[2];
#pragma unroll
  for (int stg = 0; stg < 2; ++stg) {
    const char* b = smem + stg * STAGE_BYTES;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) sp[stg].nat[ks] = b + tile_off<D>(n, 2 * ks + h);
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      sp[stg].tr0[db] = b + tr_off<D>(lane, 4 * (grp >> 1), 32 * db + 16 * (grp & 1));
      sp[stg].tr8[db] = b + tr_off<D>(lane, 8 + 4 * (grp >> 1), 32 * db + 16 * (grp & 1));
    }
    sp[stg].stat = b + 2 * TILE_BYTES + 16 * h;
  }

  f32x16 dkacc[NDB], dvacc[NDB];  // live in AGPRs
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dkacc[db][r] = 0.f; dvacc[db][r] = 0.f; }

  // The dK product of a tile's last 32-row block is left pending when the tile ends and is issued
  // at the start of the next tile, where it covers the latency of that tile's first LDS reads.
  bf16x8 qtf[2][NDB];   // Q^T fragments of the block whose dK product comes next
  bf16x8 dsf0, dsf1;    // its dS fragments
  bool pending = false; // wave-uniform
  auto flush_pending = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int m = 0; m < 2 * NDB; ++m) mfma_acc_agpr(dkacc[m % NDB], qtf[m / NDB][m % NDB], m < NDB ? dsf0 : dsf1);
  };

  const float c = p.scale_log2;

  // Unmasked tile, hand-sequenced (see mfma_asm.hpp).  The dP chain accumulates onto -delta
  // (stored negated by the delta kernel, it arrives in exactly the C layout of a 32-row block),
  // so a block's elementwise work is 16 (fma, exp2) + 8 packs for P and 16 multiplies + 8 packs
  // for dS.  P can only start after S and dS only
  // after dP, so the chains of neighbouring blocks are interleaved, which spreads that work one
  // element per MFMA over all 32 MFMAs of a block.  The two chains that accumulate in one
  // register block (S, dP: each MFMA waits for the previous one) alternate MFMA by MFMA with
  // the two that rotate over four accumulators (dK, dV).  Steady state for block b:
  //   X(b): dP(b)_m, dK(b-1)_m, m = 0..7   + P elements 0..14 of block b
  //         LDS: dO^T(b), Q rows(b+1)
  //   Y(b): dV(b)_m, S(b+1)_m,  m = 0..7   + P element 15, dS elements 0..15
  //         LDS: Q^T(b), dO rows(b+1), -lse*log2e(b+1), -delta(b+1)
  // Every operand group is requested a phase before the phase that consumes it and one or two
  // reads per MFMA, never in a burst (a wave issues in order).  X(0) has no dK (the previous
  // block's was issued in the prologue) and the last Y no S.
  // `make_next` describes the next tile (address arithmetic, all scalar); it is called behind the tile's first MFMAs,
  // which hide it: in front of them, right after the step's barrier, the matrix pipeline would wait for it.
  auto fast_tile = [&](const StagePtrs& sp_, auto make_next, auto spread_copies) __attribute__((always_inline)) {
    constexpr bool kSpread = decltype(spread_copies)::value;  // copy the next tile piece by piece between the chains
    TileCopy next;   // (described behind the first MFMAs, see below)
    static_assert(NDB == 4 || NDB == 2, "the schedule below is written for D = 128 (used) and only has to compile for 64");
    bf16x8 qn[NKS], don[NKS], dotf[2][NDB];
    f32x16 s, dp, nl, nd;   // nl: -lse*log2e of the rows of s; nd: -delta of the rows of the next dP chain
    float pr[16], ds[16];
    uint32_t pw[8], dw[8];

    auto tr_frag = [&](int blk, int tile_bytes, int m) __attribute__((always_inline)) {  // fragment m = (sblk, db)
      const int sblk = m / NDB, db = m % NDB;
      const int off = blk + 16 * sblk * ROW_BYTES + tile_bytes;
      return cat4(lds_read_tr4(sp_.tr0[db] + off), lds_read_tr4(sp_.tr8[db] + off));
    };
    auto stat4 = [&](f32x16& dst, int q4, int first_row) __attribute__((always_inline)) {  // rows first_row + 8 q4 + 4h .. +3
      const f32x4 t = *reinterpret_cast<const f32x4*>(sp_.stat + (first_row + 8 * q4) * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) dst[4 * q4 + e] = t[e];
    };
    auto p_elem = [&](int e, auto lead) __attribute__((always_inline)) {
      if (e >= 2 && (e & 1) == 0) pack_pair(pw[e / 2 - 1], pr[e - 2], pr[e - 1]);  // previous pair, one MFMA after its last exp
      softmax_elem<decltype(lead)::value>(pr[e], s[e], c, nl[e]);
    };
    auto ds_elem = [&](int e, auto lead) __attribute__((always_inline)) {
      mul_elem<decltype(lead)::value>(ds[e], pr[e], dp[e]);
      if (e & 1) pack_pair(dw[e / 2], ds[e - 1], ds[e]);
    };
    auto spread = [&](int slot_idx) __attribute__((always_inline)) {   // 4 * NB slots per tile
      if (kSpread) {
        if (STORE_DS) {
          // all copies in the first two blocks, ahead of the second block's dS stores: the step's final wait
          // then leaves only stores open (see step_fn)
          constexpr int kSlots = 8;
          if (slot_idx < kSlots) {
#pragma unroll
            for (int k = slot_idx; k < kPieces; k += kSlots) copy_piece(next, k);
          }
        } else {
          if (slot_idx < kPieces) copy_piece(next, slot_idx);
          if (slot_idx + 4 * NB < kPieces) copy_piece(next, slot_idx + 4 * NB);
        }
      }
    };

    // prologue: operands of block 0, the pending dK product in the shadow of their latency, S(0)
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qn[ks] = lds_read8(sp_.nat[ks], 0);
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) stat4(nl, q4, 0);
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) don[ks] = lds_read8(sp_.nat[ks], TILE_BYTES);
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) stat4(nd, q4, BQ);
    asm_fence();
    if (pending) flush_pending();
    asm_fence();
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      if (ks == 0) mfma_first_b_agpr(s, qn[0], kf[0]);
      else mfma_next_b_agpr(s, qn[ks], kf[ks]);
    }
    asm_fence();
    if (kSpread) next = make_next();
    asm_fence();

#pragma unroll
    for (int rb = 0; rb < NB; ++rb) {
      const int blk = 32 * rb * ROW_BYTES;
      const bool more = rb + 1 < NB;
      // ---- X(b)
#pragma unroll
      for (int m = 0; m < NKS; ++m) {
        if (m == 0) spread(4 * rb + 0);
        if (m == NKS / 2) spread(4 * rb + 1);
        if (m == 0) mfma_first_cin_b_agpr(dp, don[0], vf[0], nd);
        else mfma_next_b_agpr(dp, don[m], vf[m]);
        if (m < 2 * NDB) dotf[m / NDB][m % NDB] = tr_frag(blk, TILE_BYTES, m);
        if (rb == 0) {
          // no dK chain to alternate with: two elements per MFMA (element 14 follows in Y)
          if (m == 1) { p_elem(0, std::true_type{}); p_elem(1, std::false_type{}); }
          if (m > 1) { p_elem(2 * m - 2, std::false_type{}); p_elem(2 * m - 1, std::false_type{}); }
          if (more) qn[m] = lds_read8(sp_.nat[m], blk + 32 * ROW_BYTES);
          asm_fence();
        } else {
          if (m > 0) p_elem(2 * m - 1, std::false_type{});
          asm_fence();
          mfma_acc_agpr(dkacc[m % NDB], qtf[m / NDB][m % NDB], m < NDB ? dsf0 : dsf1);
          if (more) qn[m] = lds_read8(sp_.nat[m], blk + 32 * ROW_BYTES);
          if (m == 0) p_elem(0, std::true_type{});
          else p_elem(2 * m, std::false_type{});
          asm_fence();
        }
      }
      // ---- Y(b)
      bf16x8 pf0, pf1;
#pragma unroll
      for (int m = 0; m < 2 * NDB; ++m) {
        if (m == 0) spread(4 * rb + 2);
        if (m == NDB) spread(4 * rb + 3);
        if (m == 0) pf0 = frag_from_words(pw[0], pw[1], pw[2], pw[3]);
        if (m == NDB) pf1 = frag_from_words(pw[4], pw[5], pw[6], pw[7]);
        mfma_acc_agpr(dvacc[m % NDB], dotf[m / NDB][m % NDB], m < NDB ? pf0 : pf1);
        qtf[m / NDB][m % NDB] = tr_frag(blk, 0, m);
        if (more) {
          if (m == 0 && rb == 0) p_elem(14, std::false_type{});
          if (m == 0) softmax_elem<false>(pr[15], s[15], c, nl[15]);
          if (m > 0) ds_elem(2 * m - 1, std::false_type{});
          asm_fence();
          if (m == 0) mfma_first_b_agpr(s, qn[0], kf[0]);
          else mfma_next_b_agpr(s, qn[m], kf[m]);
          don[m] = lds_read8(sp_.nat[m], blk + 32 * ROW_BYTES + TILE_BYTES);
          if (m >= 1 && m <= 4) stat4(nl, m - 1, 32 * (rb + 1));   // element 15 has read nl[15] in slot 0
          if (m >= NKS - 4) stat4(nd, m - (NKS - 4), BQ + 32 * (rb + 1));
          if (m == 0) { pack_pair(pw[7], pr[14], pr[15]); ds_elem(0, std::true_type{}); }
          else ds_elem(2 * m, std::false_type{});
          if (m == NKS - 1) ds_elem(15, std::false_type{});
          asm_fence();
        } else {
          // last block of the tile, no S chain to alternate with: two elements per MFMA
          if (m == 0) softmax_elem<false>(pr[15], s[15], c, nl[15]);
          if (m == 1) { pack_pair(pw[7], pr[14], pr[15]); ds_elem(0, std::true_type{}); ds_elem(1, std::false_type{}); }
          if (m > 1) { ds_elem(2 * m - 2, std::false_type{}); ds_elem(2 * m - 1, std::false_type{}); }
          if (m == NKS - 1) { ds_elem(14, std::false_type{}); ds_elem(15, std::false_type{}); }
          asm_fence();
        }
      }
      dsf0 = frag_from_words(dw[0], dw[1], dw[2], dw[3]);
      dsf1 = frag_from_words(dw[4], dw[5], dw[6], dw[7]);
      if (STORE_DS) {   // read once by the next kernel: no reason to keep the lines in L2
        char* dst = ds_step + ds_lane + rb * 2048;
        __builtin_nontemporal_store(__builtin_bit_cast(u32x4, dsf0), reinterpret_cast<u32x4*>(dst));
        __builtin_nontemporal_store(__builtin_bit_cast(u32x4, dsf1), reinterpret_cast<u32x4*>(dst + 16));
      }
    }
    pending = true;
  };

  // Generic tile (diagonal, document end, D = 64): compiler-scheduled, with masks.
  // kPin keeps LDS reads from crossing the phase boundaries but lets ALU and MFMA instructions move.
  constexpr int kPin = 0x1 | 0x2 | 0x4 | 0x8 | 0x400;
  auto generic_tile = [&](const StagePtrs& sp_, const int i0) __attribute__((always_inline)) {
    if (pending) {
      flush_pending();
      mfma_result_fence();  // the compiler's own instructions may touch dkacc next
      pending = false;
    }
    bf16x8 qn[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qn[ks] = lds_read8(sp_.nat[ks], 0);
#pragma unroll
    for (int rb = 0; rb < NB; ++rb) {
      const int blk = 32 * rb * ROW_BYTES;
      bf16x8 don[NKS];
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) don[ks] = lds_read8(sp_.nat[ks], blk + TILE_BYTES);
      __builtin_amdgcn_sched_barrier(kPin);
      f32x16 s = mfma_chain_b_in_agpr<NKS>(qn, kf);
      bf16x8 dotf[2][NDB];
#pragma unroll
      for (int sblk = 0; sblk < 2; ++sblk)
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          const int off = blk + 16 * sblk * ROW_BYTES + TILE_BYTES;
          dotf[sblk][db] = cat4(lds_read_tr4(sp_.tr0[db] + off), lds_read_tr4(sp_.tr8[db] + off));
        }
      __builtin_amdgcn_sched_barrier(kPin);
      f32x16 dp = mfma_chain_b_in_agpr<NKS>(don, vf);
      bf16x8 qtg[2][NDB];
#pragma unroll
      for (int sblk = 0; sblk < 2; ++sblk)
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          const int off = blk + 16 * sblk * ROW_BYTES;
          qtg[sblk][db] = cat4(lds_read_tr4(sp_.tr0[db] + off), lds_read_tr4(sp_.tr8[db] + off));
        }
      // row statistics (-lse*log2e, -delta) of the block's 16 rows held by this lane
      f32x4 l4[4], d4[4];
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        l4[q4] = *reinterpret_cast<const f32x4*>(sp_.stat + (32 * rb + 8 * q4) * 4);
        d4[q4] = *reinterpret_cast<const f32x4*>(sp_.stat + (BQ + 32 * rb + 8 * q4) * 4);
      }
      __builtin_amdgcn_sched_barrier(kPin);
      {
        const int lim_c = p.causal ? key_rel - i0 - 32 * rb - 4 * h : -(1 << 30);  // rows below this see no key of the lane
        const int lim_e = nq - i0 - 32 * rb - 4 * h;                                // rows from here on do not exist
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int ri = 8 * (r >> 2) + (r & 3);
          if (ri < lim_c || ri >= lim_e) s[r] = -INFINITY;
        }
      }
      float pr[16];
      bf16x8 pf[2];
#pragma unroll
      for (int sblk = 0; sblk < 2; ++sblk) {
        bf16x2 pp[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int r = 8 * sblk + 2 * t;
          pr[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, l4[r >> 2][r & 3]));
          pr[r + 1] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r + 1], c, l4[r >> 2][(r & 3) + 1]));
          pp[t] = pack_bf16(pr[r], pr[r + 1]);
        }
        pf[sblk] = cat_pairs(pp[0], pp[1], pp[2], pp[3]);
      }
#pragma unroll
      for (int sblk = 0; sblk < 2; ++sblk)
#pragma unroll
        for (int db = 0; db < NDB; ++db) dvacc[db] = mfma32(dotf[sblk][db], pf[sblk], dvacc[db]);
      bf16x8 dsf[2];
#pragma unroll
      for (int sblk = 0; sblk < 2; ++sblk) {
        bf16x2 dd[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int r = 8 * sblk + 2 * t;
          dd[t] = pack_bf16(pr[r] * (dp[r] + d4[r >> 2][r & 3]), pr[r + 1] * (dp[r + 1] + d4[r >> 2][(r & 3) + 1]));
        }
        dsf[sblk] = cat_pairs(dd[0], dd[1], dd[2], dd[3]);
      }
      if (STORE_DS) {   // masked elements are exact zeros (p = exp2(-inf))
        char* dst = ds_step + ds_lane + rb * 2048;
        __builtin_nontemporal_store(__builtin_bit_cast(u32x4, dsf[0]), reinterpret_cast<u32x4*>(dst));
        __builtin_nontemporal_store(__builtin_bit_cast(u32x4, dsf[1]), reinterpret_cast<u32x4*>(dst + 16));
      }
      if (rb + 1 < NB) {
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) qn[ks] = lds_read8(sp_.nat[ks], blk + 32 * ROW_BYTES);
      }
      __builtin_amdgcn_sched_barrier(kPin);
#pragma unroll
      for (int sblk = 0; sblk < 2; ++sblk)
#pragma unroll
        for (int db = 0; db < NDB; ++db) dkacc[db] = mfma32(qtg[sblk][db], dsf[sblk], dkacc[db]);
    }
  };

  // One step = one query tile of one query head.  `slot` (compile-time) is the stage that holds it.
  int hq_idx = 0, tile_idx = 0;  // the step being computed
  auto step_fn = [&](const int st, auto slot_c) __attribute__((always_inline)) {
    constexpr int slot = decltype(slot_c)::value;
    int next_hq = hq_idx, next_tile = tile_idx + 1;
    if (next_tile == nqt) { next_tile = 0; ++next_hq; }
    const bool has_next = st + 1 < total;
    auto make_next = [&]() __attribute__((always_inline)) {
      // (the tile number is made opaque HERE: whatever depends on it is then computed behind the assembly statements
      // that precede the call, not hoisted in front of them)
      int t_next = has_next ? next_tile : tile_idx;
      asm volatile("" : "+s"(t_next));
      return describe(has_next ? next_hq : hq_idx, t_next, 1 - slot);
    };
    const bool next_full = has_next && nq - next_tile * BQ >= BQ;
    const int i0 = tile_idx * BQ;
    // Mask when a key of this wave can exceed a row of the tile (causal) or rows run past the document.
    const bool need_mask = (p.causal && wv * 32 + 31 > i0) || (i0 + BQ > nq);
    const bool fast = D == 128 && !need_mask;
    if (fast && next_full) {
      fast_tile(sp[slot], make_next, std::true_type{});
    } else {
      if (has_next) copy_all(make_next());
      if (fast) fast_tile(sp[slot], make_next, std::false_type{});
      else generic_tile(sp[slot], i0);
    }
    // The next tile's copies have landed; vector memory operations complete in issue order, and after a
    // hand-sequenced tile that copied piece by piece the six youngest are the dS stores of its last three
    // 32-row blocks, which nothing in this kernel waits for.
    if (STORE_DS && fast && next_full) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
    else async_wait_all();
    __syncthreads();
    if (STORE_DS) {
      if (next_tile == 0) { ds_first += ds_head; ds_step = ds_first; }
      else ds_step += ds_matrix_bytes(p.S / BQ, it0 + tile_idx, p.causal != 0);
    }
    hq_idx = next_hq;
    tile_idx = next_tile;
  };

  agpr_loads_wait();  // K/V fragments (and the first stage's copies) have arrived
  async_wait_all();
  __syncthreads();
  int st = 0;
  for (; st + 1 < total; st += 2) {
    step_fn(st, std::integral_constant<int, 0>{});
    step_fn(st + 1, std::integral_constant<int, 1>{});
  }
  if (st < total) step_fn(st, std::integral_constant<int, 0>{});
  if (pending) flush_pending();
  mfma_result_fence();  // the last assembly MFMAs have retired before the accumulators are read

  const int64_t key_st = key_ok ? key : tc.doc_end - 1;  // (address only formed for rows that exist)
  __bf16* dkrow = reinterpret_cast<__bf16*>(reinterpret_cast<char*>(p.dk) + kvhead + kv_row_off(key_st));
  __bf16* dvrow = reinterpret_cast<__bf16*>(reinterpret_cast<char*>(p.dv) + kvhead + kv_row_off(key_st));
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    store_block32_bf16(dkrow + 32 * db, dkacc[db], p.scale, h, key_ok);
    store_block32_bf16(dvrow + 32 * db, dvacc[db], 1.0f, h, key_ok);
  }
  }  // next item
}

// ---- dQ from a materialised dS ---------------------------------------------------------------
// When the caller's workspace has room for dS (attn_common.hpp: ds_matrix_offset), the dK/dV kernel
// stores the dS it forms anyway and dQ = scale * dS K is a plain product: one third of the dQ
// kernel's matrix work, paid for with one write and one read of dS (Hq * S^2 bytes for causal input).
// The kernel is bound by that read, so it is built as a stream: a workgroup owns TWO 128-query tiles
// (so that K is fetched once for both), 32-key stages (K rows and both tiles' dS groups, 8 KiB each) in a
// ring of three, two in flight per workgroup and two workgroups per CU.  dS arrives with the key index
// slowest, the order the dK/dV kernel holds it in, and K is key-major too, so both operands of
// dQ^T += K^T dS^T are gathered with transpose loads; wave w owns the columns of 32-query block w of both
// tiles (a permutation of the tiles' queries 32w .. 32w+31), and every K^T fragment feeds both.
template <int D>
__global__ __launch_bounds__(kThreads, 2) void attn_bwd_dq_from_ds_kernel(AttnParams p) {
  static_assert(D == 128, "the dS workspace is laid out for head dimension 128");
  constexpr int BM = 256, BN = 32, NS = 3;
  constexpr int NDB = D / 32;
  constexpr int ROW_BYTES = D * 2;
  constexpr int TILE_BYTES = BN * ROW_BYTES;   // K rows of a stage; also one tile's dS group
  constexpr int STAGE_BYTES = 3 * TILE_BYTES;  // K, dS of the first tile, dS of the second
  constexpr int PIECES = BN / 16;              // copy instructions per wave and 8 KiB
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ int scratch[8];

  __shared__ QueueState s_work;
  queue_init(p, &s_work);
  const uint32_t xcc = xcc_id();
  int skip = 0;
  for (;;) {   // persistent: one item (batch, head, pair of query tiles) per iteration (tile_queue.hpp)
  const int item = next_work(p, &s_work, xcc, skip);
  if (item < 0) break;
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wv = tid >> 6;
  const int n = lane & 31, h = lane >> 5, grp = lane >> 4;

  TileCoord tc = decode_tile<BM>(p, p.Hq, true, scratch, item, tid);
  if (!tc.valid) continue;
  const int g = tc.h / (p.Hq / p.Hkv);
  const int64_t q0 = tc.t0;
  const int ita = (int)(q0 / 128);                // first tile; the second is ita + 1 unless S ends before it
  const bool has_b = q0 + 128 < p.S;
  const bool causal = p.causal != 0;
  const int nkt_a = causal ? (ita + 1) * (128 / BN) : (int)(p.S / BN);   // stages the first tile takes part in
  const int nkt = has_b && causal ? nkt_a + 128 / BN : nkt_a;

  const int64_t kv_pitch = (int64_t)p.Hkv * D * 2;
  const char* kbase = reinterpret_cast<const char*>(p.k + g * D) + tc.b * p.kv_bstride;   // (this path takes contiguous tensors only)
  const int64_t bh = (int64_t)tc.b * p.Hq + tc.h;
  const char* sa = reinterpret_cast<const char*>(p.ds) + ds_matrix_offset(p.S / 128, bh, ita, causal);
  const char* sb = has_b ? sa + ds_matrix_bytes(p.S / 128, ita, causal) : sa;   // (without a second tile: valid memory, never used)

  const uint32_t lds0 = lds_address(smem);
  AsyncTile<D> ldk;
  ldk.init(tid, kv_pitch);
  const int wave_u = ldk.wave;
  // Every stage issues the same six instructions per wave, so that the waits below can count them: past the
  // first tile's last stage its copy repeats that stage (8 KiB that nobody reads, four times per item).
  auto issue = [&](const int kt, const int slot) __attribute__((always_inline)) {
    const uint32_t dst = lds0 + slot * STAGE_BYTES;
    const int kta = kt < nkt_a ? kt : nkt_a - 1;
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
      const int piece = (i * 4 + wave_u) * 1024;
      ldk.load_full_piece(dst, kbase + (int64_t)kt * BN * kv_pitch, i);
      // the 32-key groups of dS, as they lie in memory
      async_copy16_stream((uint32_t)lane * 16u, sa + (int64_t)kta * TILE_BYTES + piece, dst + TILE_BYTES + piece);
      async_copy16_stream((uint32_t)lane * 16u, sb + (int64_t)kt * TILE_BYTES + piece, dst + 2 * TILE_BYTES + piece);
    }
  };
#pragma unroll
  for (int t = 0; t < NS - 1; ++t) issue(t, t);

  const char* tr_k0[NDB];   // K^T fragments: keys 4 (grp / 2) .. +3 and 8 + ..., columns 32 db + lane % 32
  const char* tr_k8[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    tr_k0[db] = smem + tr_off<D>(lane, 4 * (grp >> 1), 32 * db + 16 * (grp & 1));
    tr_k8[db] = smem + tr_off<D>(lane, 8 + 4 * (grp >> 1), 32 * db + 16 * (grp & 1));
  }
  // dS^T fragments of the wave's columns: lane L of a 16-lane group addresses key r0 + L / 4, values 4 (L % 4) .. +3
  // of half-wave slot hh = grp & 1 (see the workspace layout in attn_common.hpp)
  const int hh = grp & 1, l16 = lane & 15;
  const char* tr_s0 = smem + TILE_BYTES + wv * 2048 + hh * 1024 + ((((4 * (grp >> 1)) ^ (4 * hh)) + (l16 >> 2)) << 5) + ((l16 & 3) << 3);
  const char* tr_s8 = smem + TILE_BYTES + wv * 2048 + hh * 1024 + ((((8 + 4 * (grp >> 1)) ^ (4 * hh)) + (l16 >> 2)) << 5) + ((l16 & 3) << 3);

  f32x16 acc_a[NDB], acc_b[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc_a[db][r] = 0.f; acc_b[db][r] = 0.f; }

  // the copies of stage t+1 have landed when at most the 3 * PIECES * (NS - 2) instructions issued after them are open
  auto wait_next = [&](const bool issued) __attribute__((always_inline)) {
    static_assert(3 * PIECES * (NS - 2) == 6, "the immediate below");
    if (issued) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
    else async_wait_all();
  };
  auto step = [&](const int kt, auto slot_c) __attribute__((always_inline)) {
    constexpr int slot = decltype(slot_c)::value;
    const bool more = kt + NS - 1 < nkt;
    if (more) issue(kt + NS - 1, (slot + NS - 1) % NS);   // the stage consumed in the previous step
    const bool do_a = kt < nkt_a;
#pragma unroll
    for (int ks = 0; ks < BN / 16; ++ks) {
      const int off = slot * STAGE_BYTES + 16 * ks * ROW_BYTES;
      const int soff = slot * STAGE_BYTES + 16 * ks * 32;   // 32 bytes per key inside a (block, half-wave) slot group
      bf16x8 ktf[NDB];
#pragma unroll
      for (int db = 0; db < NDB; ++db) ktf[db] = cat4(lds_read_tr4(tr_k0[db] + off), lds_read_tr4(tr_k8[db] + off));
      if (do_a) {
        const bf16x8 dsa = cat4(lds_read_tr4(tr_s0 + soff), lds_read_tr4(tr_s8 + soff));
#pragma unroll
        for (int db = 0; db < NDB; ++db) acc_a[db] = mfma32(ktf[db], dsa, acc_a[db]);
      }
      if (has_b) {
        const bf16x8 dsb = cat4(lds_read_tr4(tr_s0 + soff + TILE_BYTES), lds_read_tr4(tr_s8 + soff + TILE_BYTES));
#pragma unroll
        for (int db = 0; db < NDB; ++db) acc_b[db] = mfma32(ktf[db], dsb, acc_b[db]);
      }
    }
    wait_next(more);
    __syncthreads();
  };

  wait_next(true);
  __syncthreads();
  int kt = 0;
  for (; kt + NS <= nkt; kt += NS) {
    step(kt, std::integral_constant<int, 0>{});
    step(kt + 1, std::integral_constant<int, 1>{});
    step(kt + 2, std::integral_constant<int, 2>{});
  }
  if (kt < nkt) step(kt, std::integral_constant<int, 0>{});
  if (kt + 1 < nkt) step(kt + 1, std::integral_constant<int, 1>{});

  // column 32 wv + n of a tile is its query 32 wv + 8 (e / 4) + 4 hh + e % 4 with hh = n / 16, e = n % 16
  const int e = n & 15;
  const int64_t row = q0 + 32 * wv + 8 * (e >> 2) + 4 * (n >> 4) + (e & 3);
  __bf16* drow = p.dq + (((int64_t)tc.b * p.S + row) * p.Hq + tc.h) * D;
#pragma unroll
  for (int db = 0; db < NDB; ++db) store_block32_bf16(drow + 32 * db, acc_a[db], p.scale, h, true);
  drow += (int64_t)128 * p.Hq * D;
#pragma unroll
  for (int db = 0; db < NDB; ++db) store_block32_bf16(drow + 32 * db, acc_b[db], p.scale, h, has_b);
  }  // next item
}

// Work-queue counters of the two main kernels inside the workspace's counter area (in 4-byte units).
constexpr int kCountersDq = 0, kCountersDkdv = kQueueBytes / 4;
constexpr int kDqWaves = 8;   // waves per workgroup of the recomputing dQ kernel at head dimension 128 (four: 2 % slower)

template <int D>
static int launch_bwd_d(AttnParams p, int phases, hipStream_t st) {
  hipError_t e;
  if (phases & 1) {  // delta
    AttnParams a = p;
    a.tiles = kDeltaTokens;
    while (a.tiles > 1 && (size_t)p.Hq * a.tiles * sizeof(float) > 48 * 1024) a.tiles /= 2;
    const size_t smem = (size_t)p.Hq * a.tiles * sizeof(float);
    if (smem > 48 * 1024) return kErrShape;   // more than 12288 query heads per GPU
    int64_t grid = ceil_div(p.S, a.tiles) * p.B;
    if (grid >= ((int64_t)1 << 31)) return kErrShape;
    attn_bwd_delta_kernel<D><<<dim3((unsigned)grid), dim3(kThreads), smem, st>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e);
  }
  const bool cleared_by_delta = (phases & 1) != 0;   // the delta kernel of this call clears both queues' counters
  // With room for dS in the workspace (p.ds), dK/dV runs first and stores it, and dQ is one product.
  const bool from_ds = p.ds != nullptr;
  auto dq_phase = [&]() -> int {
    int64_t tiles = tiles_per_head(p.S, from_ds ? 256 : 128, p.cu, p.num_docs);
    int64_t items = tiles * p.B * p.Hq;
    if (items >= ((int64_t)1 << 31)) return kErrShape;
    AttnParams a = p;
    a.tiles = (int32_t)tiles;
    if constexpr (D == 128) {
      if (from_ds) {
        constexpr int smem = 3 * 3 * 32 * D * 2;
        static KernelSetup setup;
        int per_cu = 1;
        int rc = kernel_setup(setup, attn_bwd_dq_from_ds_kernel<D>, smem, &per_cu);
        if (rc) return rc;
        const QueueLaunch ql = tile_queue_prepare(a, p.ws_counters + kCountersDq, items, a.Hq, per_cu, st, cleared_by_delta);
        if (ql.err != hipSuccess) return hip_fail(ql.err);
        attn_bwd_dq_from_ds_kernel<D><<<dim3((unsigned)ql.grid), dim3(kThreads), smem, st>>>(a);
        if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e);
        return 0;
      }
    }
    auto recompute = [&](auto waves_c) -> int {
      constexpr int W = decltype(waves_c)::value;
      constexpr int smem = DqCfg<W>::template smem_bytes<D>();
      static KernelSetup setup;
      int per_cu = 1;
      int rc = kernel_setup(setup, attn_bwd_dq_kernel<D, W>, smem, &per_cu, 64 * W);
      if (rc) return rc;
      tiles = tiles_per_head(p.S, DqCfg<W>::BM, p.cu, p.num_docs);
      items = tiles * p.B * p.Hq;
      a.tiles = (int32_t)tiles;
      const QueueLaunch ql = tile_queue_prepare(a, p.ws_counters + kCountersDq, items, a.Hq, per_cu, st, cleared_by_delta);
      if (ql.err != hipSuccess) return hip_fail(ql.err);
      attn_bwd_dq_kernel<D, W><<<dim3((unsigned)ql.grid), dim3(64 * W), smem, st>>>(a);
      if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e);
      return 0;
    };
    if constexpr (D == 128) {
      if (!dq_prefers_128_rows(ceil_div(p.S, DqCfg<kDqWaves>::BM) * p.B * p.Hq, p.S, p.cu != nullptr)) return recompute(std::integral_constant<int, kDqWaves>{});
    }
    return recompute(std::integral_constant<int, 4>{});
  };
  auto dkdv_phase = [&](auto store_c, auto chunked_c) -> int {
    constexpr bool kStore = decltype(store_c)::value, kChunked = decltype(chunked_c)::value;
    constexpr int smem = DkdvCfg<D>::SMEM_BYTES;
    static KernelSetup setup;
    int per_cu = 1;
    int rc = kernel_setup(setup, attn_bwd_dkdv_kernel<D, kStore, kChunked>, smem, &per_cu);
    if (rc) return rc;
    int64_t tiles = tiles_per_head(p.S, 128, p.cu, p.num_docs);
    int64_t items = tiles * p.B * p.Hkv;
    if (items >= ((int64_t)1 << 31)) return kErrShape;
    AttnParams a = p;
    a.tiles = (int32_t)tiles;
    const QueueLaunch ql = tile_queue_prepare(a, p.ws_counters + kCountersDkdv, items, a.Hkv, per_cu, st, cleared_by_delta);
    if (ql.err != hipSuccess) return hip_fail(ql.err);
    attn_bwd_dkdv_kernel<D, kStore, kChunked><<<dim3((unsigned)ql.grid), dim3(kThreads), smem, st>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e);
    return 0;
  };
  const bool chunked = p.tok_shift < 63;
  int rc = 0;
  if (from_ds) {
    if constexpr (D == 128) {
      if ((phases & 4) && (rc = dkdv_phase(std::true_type{}, std::false_type{}))) return rc;
    }
    if ((phases & 2) && (rc = dq_phase())) return rc;
  } else {
    if ((phases & 2) && (rc = dq_phase())) return rc;
    if ((phases & 4) && (rc = chunked ? dkdv_phase(std::false_type{}, std::true_type{}) : dkdv_phase(std::false_type{}, std::false_type{}))) return rc;
  }
  return 0;
}

int launch_bwd(AttnParams p, int D, int phases, hipStream_t st) {
  return D == 64 ? launch_bwd_d<64>(p, phases, st) : launch_bwd_d<128>(p, phases, st);
}

}  // namespace ie
