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
#include "attn_common.hpp"
#include "launch.hpp"

namespace ie {

template <int D>
__global__ __launch_bounds__(kThreads, 2) void attn_fwd_kernel(AttnParams p) {
  constexpr int BM = 128, BN = 64;
  constexpr int NKS = D / 16;  // k-steps of the QK^T product
  constexpr int NDB = D / 32;  // 32-wide blocks of the head dimension in O^T
  constexpr int TILE_BYTES = BN * D * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  // stage s: K at smem + s * 2 * TILE_BYTES, V right after it
  __shared__ int scratch[8];

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int n = lane & 31, h = lane >> 5;

  TileCoord tc = decode_tile<BM>(p, p.Hq, true, scratch);
  if (!tc.valid) return;
  const int g = tc.h / (p.Hq / p.Hkv);
  const int64_t q0 = tc.t0;
  const int64_t q_end = (q0 + BM < tc.doc_end) ? q0 + BM : tc.doc_end;  // one past the tile's last row
  const int64_t k_begin = tc.doc_begin;
  const int64_t k_end = p.causal ? q_end : tc.doc_end;
  const int nkt = (int)((k_end - k_begin + BN - 1) / BN);

  const int64_t q_stride = (int64_t)p.Hq * D, kv_stride = (int64_t)p.Hkv * D;
  const __bf16* qbase = p.q + ((int64_t)tc.b * p.S * p.Hq + tc.h) * D;
  const __bf16* kbase = p.k + ((int64_t)tc.b * p.S * p.Hkv + g) * D;
  const __bf16* vbase = p.v + ((int64_t)tc.b * p.S * p.Hkv + g) * D;

  // This lane's query row (clamped into the tile so that out-of-range lanes repeat the last row).
  int64_t row = q0 + wv * 32 + n;
  const bool row_ok = row < q_end;
  if (!row_ok) row = q_end - 1;

  // Q fragments: B operand of S^T = K Q^T, column n = query, k = head-dim index.
  bf16x8 qf[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks)
    qf[ks] = *reinterpret_cast<const bf16x8*>(qbase + row * q_stride + ks * 16 + h * 8);

  // LDS offsets that do not change over the loop.
  int k_off[2][NKS];  // K tile, A operand: row = key 32j + n, chunk = 2ks + h
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) k_off[j][ks] = tile_off<D>(32 * j + n, 2 * ks + h);
  // V tile, transpose loads: d block db, key group (j, s, a): rows 32j + 16s + 8a + 4h .. +3
  const int grp = lane >> 4;  // 16-lane group: grp % 2 picks the 16-column half, grp / 2 == h
  int v_off[NDB];             // for rows starting at 4h; other row groups add a multiple of 8 rows
#pragma unroll
  for (int db = 0; db < NDB; ++db) v_off[db] = tr_off<D>(lane, 4 * (grp >> 1), 32 * db + 16 * (grp & 1));
  // Row r0 + 8x keeps the same swizzle when 8x is a multiple of 16 only; so precompute per (x) instead.
  // swz(r) depends on r & 15, and row groups differ by multiples of 8, so two variants suffice.
  int v_off8[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) v_off8[db] = tr_off<D>(lane, 8 + 4 * (grp >> 1), 32 * db + 16 * (grp & 1));

  TileRegs<BN, D> kr, vr;
  tile_load<BN, D>(kr, kbase, kv_stride, k_begin, k_end - 1, tid);
  tile_load<BN, D>(vr, vbase, kv_stride, k_begin, k_end - 1, tid);
  tile_store<BN, D>(kr, smem, tid);
  tile_store<BN, D>(vr, smem + TILE_BYTES, tid);
  __syncthreads();

  const float c = p.scale_log2;
  float m = -INFINITY;  // running row maximum of the raw (unscaled) scores
  float l = 0.f;        // this lane's share of the row sum (its half of the keys)
  f32x16 oacc[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;

  const int64_t wave_row_min = q0 + wv * 32;
  for (int kt = 0; kt < nkt; ++kt) {
    const int64_t kb = k_begin + (int64_t)kt * BN;
    const char* ks_lds = smem + (kt & 1) * 2 * TILE_BYTES;
    const char* vs_lds = ks_lds + TILE_BYTES;
    const bool more = kt + 1 < nkt;
    if (more) {
      tile_load<BN, D>(kr, kbase, kv_stride, kb + BN, k_end - 1, tid);
      tile_load<BN, D>(vr, vbase, kv_stride, kb + BN, k_end - 1, tid);
    }

    // S^T blocks: rows = keys kb + 32j .. +31, column = this lane's query
    f32x16 s[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[j][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) s[j] = mfma32(lds_read8(ks_lds, k_off[j][ks]), qf[ks], s[j]);
    }

    // Mask: only tiles that reach past the wave's first row (causal) or past the last key.
    const bool need_mask = (p.causal && kb + BN - 1 > wave_row_min) || (kb + BN > k_end);
    if (need_mask) {
      const int64_t lim = p.causal ? (row < k_end - 1 ? row : k_end - 1) : k_end - 1;  // last visible key
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int64_t key = kb + 32 * j + 8 * (r >> 2) + 4 * h + (r & 3);
          if (key > lim) s[j][r] = -INFINITY;
        }
    }

    float mx = s[0][0];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[j][r]);
    mx = halfwave_max(mx);
    const float m_new = fmaxf(m, mx);
    if (__builtin_amdgcn_ballot_w64(m_new > m) != 0) {  // some row's maximum moved: rescale
      const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);
      l *= alpha;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
    m = m_new;
    const float mc = m * c;
    bf16x8 pf[2][2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s[j][r], c, -mc));
        l += e;
        pf[j][r >> 3][r & 7] = (__bf16)e;
      }

    // O^T += V^T P^T
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int sblk = 0; sblk < 2; ++sblk) {
        const int rowbytes = (32 * j + 16 * sblk) * (D * 2);
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          bf16x4 lo = lds_read_tr4(vs_lds + rowbytes + v_off[db]);
          bf16x4 hi = lds_read_tr4(vs_lds + rowbytes + v_off8[db]);
          oacc[db] = mfma32(cat4(lo, hi), pf[j][sblk], oacc[db]);
        }
      }

    if (more) {
      char* nk = smem + ((kt + 1) & 1) * 2 * TILE_BYTES;
      tile_store<BN, D>(kr, nk, tid);
      tile_store<BN, D>(vr, nk + TILE_BYTES, tid);
    }
    __syncthreads();
  }

  // Epilogue: normalise, write O (bf16) and LSE (natural log).
  const float l_full = halfwave_sum(l);
  const float inv_l = 1.0f / l_full;
  if (row_ok) {
    __bf16* orow = p.o_out + ((int64_t)tc.b * p.S * p.Hq + tc.h) * D + row * q_stride;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        bf16x4 w;
#pragma unroll
        for (int t = 0; t < 4; ++t) w[t] = (__bf16)(oacc[db][4 * q4 + t] * inv_l);
        *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * q4 + 4 * h) = w;
      }
    if (h == 0) p.lse_out[((int64_t)tc.b * p.Hq + tc.h) * p.S + row] = (m * c + __builtin_amdgcn_logf(l_full)) * kLn2;
  }
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
  return D == 64 ? launch_fwd_d<64>(p, st) : launch_fwd_d<128>(p, st);
}

}  // namespace ie
