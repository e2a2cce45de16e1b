// Forward kernel: O = softmax(scale * Q K^T + mask) V and the per-row log-sum-exp, one
// workgroup per (batch, head, 128-query tile), streaming 64-key tiles of K and V through
// double-buffered LDS (fused attention of Sec. 2.1 / Sec. 4.2, recast for CDNA4).
//
// Each of the 4 wavefronts owns 32 query rows and keeps its Q fragments in registers.
// Scores are produced TRANSPOSED, S^T = K Q^T, so that one lane holds one query column:
// the row maximum and row sum are then reductions over the lane's own registers plus
// one half-wave swap, and the exponentiated scores are already in the B-operand layout
// of the second product O^T = V^T P^T, whose A operand (V^T) is gathered from the
// row-major V tile by LDS transpose loads.
#include <type_traits>

#include "attn_common.hpp"
#include "launch.hpp"

namespace ie {

template <int D>
__global__ __launch_bounds__(kThreads, 2) void attn_fwd_kernel(AttnParams p) {
  constexpr int BM = 128, BN = 64;
  constexpr int NKS = D / 16;  // k-steps of the QK^T product
  constexpr int NDB = D / 32;  // 32-wide blocks of the head dimension in O^T
  constexpr int TILE_BYTES = BN * D * 2;
  constexpr int STAGE_BYTES = 2 * TILE_BYTES;  // K tile, then V tile
  constexpr int ROW_BYTES = D * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];  // 2 stages
  __shared__ int scratch[8];

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int n = lane & 31, h = lane >> 5, grp = lane >> 4;

  TileCoord tc = decode_tile<BM>(p, p.Hq, true, scratch, blockIdx.x, tid);
  if (!tc.valid) return;
  const int g = tc.h / (p.Hq / p.Hkv);
  const int64_t q0 = tc.t0;
  const int64_t q_end = (q0 + BM < tc.doc_end) ? q0 + BM : tc.doc_end;  // one past the tile's last row
  const int64_t k_begin = tc.doc_begin;
  const int64_t k_end = p.causal ? q_end : tc.doc_end;
  const int nk = (int)(k_end - k_begin);  // visible keys of the tile (before the per-row causal cut)
  const int nkt = (nk + BN - 1) / BN;     // key tiles
  const int nfull = nk / BN;              // of which complete

  const int64_t q_stride = (int64_t)p.Hq * D;
  const int64_t kv_pitch = (int64_t)p.Hkv * D * 2;  // bytes between consecutive tokens of one kv head
  const char* qbase = reinterpret_cast<const char*>(p.q + tc.h * D) + tc.b * p.q_bstride;
  const char* kbase = reinterpret_cast<const char*>(p.k + g * D) + tc.b * p.kv_bstride;   // key tile kt starts at token k_begin + kt * BN
  const char* vbase = reinterpret_cast<const char*>(p.v + g * D) + tc.b * p.kv_bstride;
  auto key_tile_off = [&](const int kt) __attribute__((always_inline)) { return tok_off(p, k_begin + (int64_t)kt * BN, kv_pitch); };

  const uint32_t lds0 = lds_address(smem);
  AsyncTile<D> ld;
  ld.init(tid, kv_pitch);
  ld.load(lds0, kbase + key_tile_off(0), nk);
  ld.load(lds0 + TILE_BYTES, vbase + key_tile_off(0), nk);

  // This lane's query row (clamped into the tile so that out-of-range lanes repeat the last row).
  int64_t row = q0 + wv * 32 + n;
  const bool row_ok = row < q_end;
  if (!row_ok) row = q_end - 1;
  const int row_rel = (int)(row - k_begin);  // position of the row among the document's keys

  // Q fragments: B operand of S^T = K Q^T, column n = query, k = head-dim index.
  bf16x8 qf[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks)
    qf[ks] = *reinterpret_cast<const bf16x8*>(qbase + tok_off(p, row, q_stride * 2) + (ks * 16 + h * 8) * 2);

  // Per-lane LDS addresses inside stage 0; stage, tile and row-block offsets are immediates.
  const char* k_ptr[NKS];  // K tile, A operand: row = key n (+32 for the second block), chunk = 2ks + h
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) k_ptr[ks] = smem + tile_off<D>(n, 2 * ks + h);
  // V tile, transpose loads: rows 4h..4h+3 (v_ptr0) and 8+4h.. (v_ptr8) of each 16-key group
  const char* v_ptr0[NDB];
  const char* v_ptr8[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    v_ptr0[db] = smem + TILE_BYTES + tr_off<D>(lane, 4 * (grp >> 1), 32 * db + 16 * (grp & 1));
    v_ptr8[db] = smem + TILE_BYTES + tr_off<D>(lane, 8 + 4 * (grp >> 1), 32 * db + 16 * (grp & 1));
  }

  const float c = p.scale_log2;
  // The running reference m only moves when a row maximum exceeds it by more than kSlack (in
  // log2 units): exponentials then stay below 2^kSlack, the final normalisation by l is exact
  // either way, and the accumulator is rescaled only a handful of times per row.
  constexpr float kSlack = 8.0f;
  const float slack_raw = kSlack / c;
  float m = -INFINITY;  // reference maximum, raw (unscaled) score units
  float l = 0.f;        // this lane's share of the row sum (its half of the keys)
  f32x16 oacc[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;

  const int wave_row_min = (int)(q0 - k_begin) + wv * 32;

  // One 64-key LDS tile is consumed as two 32-key blocks, each with its own softmax update.
  // `stage` is the byte offset of the stage holding tile kt; FULL_NEXT says that tile kt+1
  // exists and is complete (the common case, no per-lane address arithmetic).
  auto tile_step = [&](const int kt, const int stage, auto full_next) __attribute__((always_inline)) {
    const int kb = kt * BN;  // first key of the tile, relative to k_begin
    const uint32_t next_lds = lds0 + (STAGE_BYTES - stage);
    if (full_next) {
      ld.load_full(next_lds, kbase + key_tile_off(kt + 1));
      ld.load_full(next_lds + TILE_BYTES, vbase + key_tile_off(kt + 1));
    } else if (kt + 1 < nkt) {
      ld.load(next_lds, kbase + key_tile_off(kt + 1), nk - kb - BN);
      ld.load(next_lds + TILE_BYTES, vbase + key_tile_off(kt + 1), nk - kb - BN);
    }
    // Mask: only tiles that reach past the wave's first row (causal) or past the last key.
    const bool need_mask = (p.causal && kb + BN - 1 > wave_row_min) || (kb + BN > nk);
    const int lim = (p.causal ? row_rel : nk - 1) - kb - 4 * h;  // last visible key relative to the lane's first key

#pragma unroll
    for (int j = 0; j < 2; ++j) {
      // S^T block: rows = keys kb + 32j .. +31, column = this lane's query
      f32x16 s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        s = mfma32(lds_read8(k_ptr[ks], stage + 32 * j * ROW_BYTES), qf[ks], s);
      }

      // V^T fragments of this block: requested now, consumed after the exponentials
      bf16x8 vfrag[2][NDB];
#pragma unroll
      for (int sblk = 0; sblk < 2; ++sblk)
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          const int off = stage + (32 * j + 16 * sblk) * ROW_BYTES;
          vfrag[sblk][db] = cat4(lds_read_tr4(v_ptr0[db] + off), lds_read_tr4(v_ptr8[db] + off));
        }

      if (need_mask) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (32 * j + 8 * (r >> 2) + (r & 3) > lim) s[r] = -INFINITY;
      }
      float mx = s[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
      mx = halfwave_max(mx);
      if (__builtin_amdgcn_ballot_w64(mx > m + slack_raw) != 0) {  // some row outgrew its reference
        const float m_new = fmaxf(m, mx);
        const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);
        m = m_new;
        l *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
      }
      const float mc = m * c;
      bf16x8 pf[2];
#pragma unroll
      for (int sblk = 0; sblk < 2; ++sblk) {
        bf16x2 pr[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[8 * sblk + 2 * t], c, -mc));
          const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[8 * sblk + 2 * t + 1], c, -mc));
          pr[t] = pack_bf16(e0, e1);
          l += e0 + e1;  // fp32 sum of the unrounded exponentials: lse needs more than bf16 precision
        }
        pf[sblk] = cat_pairs(pr[0], pr[1], pr[2], pr[3]);
      }
      // O^T += V^T P^T
#pragma unroll
      for (int sblk = 0; sblk < 2; ++sblk)
#pragma unroll
        for (int db = 0; db < NDB; ++db) oacc[db] = mfma32(vfrag[sblk][db], pf[sblk], oacc[db]);
    }
    async_wait_all();  // the copies of the next stage have landed ...
    __syncthreads();   // ... for every wave, and every wave is done reading this stage
  };

#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) consume(qf[ks]);
  async_wait_all();
  __syncthreads();
  int kt = 0;
  // steady state: two tiles per trip so that the stage offsets are compile-time constants
  for (; kt + 2 < nfull; kt += 2) {
    tile_step(kt, 0, std::true_type{});
    tile_step(kt + 1, STAGE_BYTES, std::true_type{});
  }
  for (; kt < nkt; ++kt) tile_step(kt, (kt & 1) * STAGE_BYTES, std::false_type{});

  // Epilogue: normalise, write O (bf16) and LSE (natural log).
  const float l_full = halfwave_sum(l);
  const float inv_l = 1.0f / l_full;
  __bf16* orow = p.o_out + ((int64_t)tc.b * p.S * p.Hq + tc.h) * D + row * q_stride;
#pragma unroll
  for (int db = 0; db < NDB; ++db) store_block32_bf16(orow + 32 * db, oacc[db], inv_l, h, row_ok);
  if (row_ok && h == 0) p.lse_out[((int64_t)tc.b * p.Hq + tc.h) * p.S + row] = (m * c + __builtin_amdgcn_logf(l_full)) * kLn2;
}

template <int D>
static int launch_fwd_d(AttnParams p, hipStream_t st) {
  constexpr int smem = 2 * 2 * 64 * D * 2;  // two stages of a K and a V tile
  int rc = set_smem(attn_fwd_kernel<D>, smem);
  if (rc) return rc;
  int64_t tiles = tiles_per_head(p.S, 128, p.cu, p.num_docs);
  int64_t grid = tiles * p.B * p.Hq;
  if (grid >= ((int64_t)1 << 31)) return kErrShape;
  p.tiles = (int32_t)tiles;
  attn_fwd_kernel<D><<<dim3((unsigned)grid), dim3(kThreads), smem, st>>>(p);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? 0 : hip_fail(e);
}

int launch_fwd(AttnParams p, int D, hipStream_t st) {
  if (D == 128 && !fwd_prefers_128_rows(ceil_div(p.S, 256) * p.B * p.Hq, p.S, p.cu != nullptr)) return launch_fwd_wide(p, st);
  return D == 64 ? launch_fwd_d<64>(p, st) : launch_fwd_d<128>(p, st);
}

}  // namespace ie
