// Backward kernels.  The probabilities are recomputed from the saved log-sum-exp (the
// fused kernel's selective recomputation, Sec. 3.1), and the five products of the
// backward pass (Sec. 4.3: backward is the compute-heavier direction) are split over two
// kernels so that each output has exactly one owner and nothing is accumulated through
// memory:
//   attn_bwd_delta : delta_i = <dO_i, O_i>                              (HBM-bound)
//   attn_bwd_dq    : query-stationary, like the forward: S^T = K Q^T, dP^T = V dO^T,
//                    dS^T = P^T o (dP^T - delta), dQ^T += K^T dS^T
//   attn_bwd_dkdv  : key-stationary: S = Q K^T, dP = dO V^T, dV^T += dO^T P,
//                    dK^T += Q^T dS, looping over the query heads of the kv head's group
// In both main kernels the elementwise results leave the first products in the C layout
// (one column per lane, rows over registers) with the NEXT contraction index on the
// rows, so they feed the following MFMA from registers; the transposed operands
// (K^T, dO^T, Q^T) are gathered from row-major LDS tiles with transpose loads.
#include "attn_common.hpp"
#include "launch.hpp"

namespace ie {

// ---- delta = rowsum(dO o O) ------------------------------------------------------------
// One (batch, token, head) row of D bf16 per group of D/8 lanes; rows are walked so that
// consecutive groups take consecutive tokens of one head, which makes the [B,Hq,S]
// writes contiguous while every read is a full row (D*2 contiguous bytes).
template <int D>
__global__ __launch_bounds__(kThreads) void attn_bwd_delta_kernel(AttnParams p) {
  constexpr int LPR = D / 8;               // lanes per row
  constexpr int RPB = kThreads / LPR;      // rows per pass of the workgroup
  constexpr int PASSES = 8;
  const int tid = threadIdx.x;
  const int sub = tid % LPR, rloc = tid / LPR;
  const int64_t blocks_per_head = (p.S + RPB * PASSES - 1) / (RPB * PASSES);
  const int64_t hh = blockIdx.x / blocks_per_head;  // b * Hq + h
  const int64_t blk = blockIdx.x % blocks_per_head;
  const int64_t b = hh / p.Hq, h = hh % p.Hq;
#pragma unroll
  for (int ps = 0; ps < PASSES; ++ps) {
    const int64_t i = (blk * PASSES + ps) * RPB + rloc;
    float acc = 0.f;
    if (i < p.S) {
      const int64_t off = ((b * p.S + i) * p.Hq + h) * D + sub * 8;
      bf16x8 x = *reinterpret_cast<const bf16x8*>(p.o + off);
      bf16x8 y = *reinterpret_cast<const bf16x8*>(p.dout + off);
#pragma unroll
      for (int t = 0; t < 8; ++t) acc = __builtin_fmaf((float)x[t], (float)y[t], acc);
    }
#pragma unroll
    for (int s = LPR / 2; s >= 1; s >>= 1) acc += __shfl_xor(acc, s, 64);
    if (sub == 0 && i < p.S) p.delta[hh * p.S + i] = acc;
  }
}

// ---- dQ ----------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kThreads, 2) void attn_bwd_dq_kernel(AttnParams p) {
  constexpr int BM = 128, BN = 64;
  constexpr int NKS = D / 16, NDB = D / 32;
  constexpr int TILE_BYTES = BN * D * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ int scratch[8];

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int n = lane & 31, h = lane >> 5, grp = lane >> 4;

  TileCoord tc = decode_tile<BM>(p, p.Hq, true, scratch);
  if (!tc.valid) return;
  const int g = tc.h / (p.Hq / p.Hkv);
  const int64_t q0 = tc.t0;
  const int64_t q_end = (q0 + BM < tc.doc_end) ? q0 + BM : tc.doc_end;
  const int64_t k_begin = tc.doc_begin;
  const int64_t k_end = p.causal ? q_end : tc.doc_end;
  const int nkt = (int)((k_end - k_begin + BN - 1) / BN);

  const int64_t q_stride = (int64_t)p.Hq * D, kv_stride = (int64_t)p.Hkv * D;
  const int64_t qhead = ((int64_t)tc.b * p.S * p.Hq + tc.h) * D;
  const __bf16* kbase = p.k + ((int64_t)tc.b * p.S * p.Hkv + g) * D;
  const __bf16* vbase = p.v + ((int64_t)tc.b * p.S * p.Hkv + g) * D;

  int64_t row = q0 + wv * 32 + n;
  const bool row_ok = row < q_end;
  if (!row_ok) row = q_end - 1;

  bf16x8 qf[NKS], dof[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    qf[ks] = *reinterpret_cast<const bf16x8*>(p.q + qhead + row * q_stride + ks * 16 + h * 8);
    dof[ks] = *reinterpret_cast<const bf16x8*>(p.dout + qhead + row * q_stride + ks * 16 + h * 8);
  }
  const int64_t stat = ((int64_t)tc.b * p.Hq + tc.h) * p.S + row;
  const float lse2 = p.lse[stat] * kLog2e;
  const float delta = p.delta[stat];

  int nat_off[2][NKS];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) nat_off[j][ks] = tile_off<D>(32 * j + n, 2 * ks + h);
  int tr0[NDB], tr8[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    tr0[db] = tr_off<D>(lane, 4 * (grp >> 1), 32 * db + 16 * (grp & 1));
    tr8[db] = tr_off<D>(lane, 8 + 4 * (grp >> 1), 32 * db + 16 * (grp & 1));
  }

  TileRegs<BN, D> kr, vr;
  tile_load<BN, D>(kr, kbase, kv_stride, k_begin, k_end - 1, tid);
  tile_load<BN, D>(vr, vbase, kv_stride, k_begin, k_end - 1, tid);
  tile_store<BN, D>(kr, smem, tid);
  tile_store<BN, D>(vr, smem + TILE_BYTES, tid);
  __syncthreads();

  const float c = p.scale_log2;
  f32x16 acc[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

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
    const bool need_mask = (p.causal && kb + BN - 1 > wave_row_min) || (kb + BN > k_end);
    const int64_t lim = p.causal ? (row < k_end - 1 ? row : k_end - 1) : k_end - 1;

#pragma unroll
    for (int j = 0; j < 2; ++j) {
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) s = mfma32(lds_read8(ks_lds, nat_off[j][ks]), qf[ks], s);
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) dp = mfma32(lds_read8(vs_lds, nat_off[j][ks]), dof[ks], dp);
      if (need_mask) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int64_t key = kb + 32 * j + 8 * (r >> 2) + 4 * h + (r & 3);
          if (key > lim) s[r] = -INFINITY;
        }
      }
      bf16x8 dsf[2];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -lse2));
        dsf[r >> 3][r & 7] = (__bf16)(pr * (dp[r] - delta));
      }
      // dQ^T += K^T dS^T over this block's 32 keys
#pragma unroll
      for (int sblk = 0; sblk < 2; ++sblk) {
        const int rowbytes = (32 * j + 16 * sblk) * (D * 2);
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          bf16x4 lo = lds_read_tr4(ks_lds + rowbytes + tr0[db]);
          bf16x4 hi = lds_read_tr4(ks_lds + rowbytes + tr8[db]);
          acc[db] = mfma32(cat4(lo, hi), dsf[sblk], acc[db]);
        }
      }
    }

    if (more) {
      char* nk = smem + ((kt + 1) & 1) * 2 * TILE_BYTES;
      tile_store<BN, D>(kr, nk, tid);
      tile_store<BN, D>(vr, nk + TILE_BYTES, tid);
    }
    __syncthreads();
  }

  if (row_ok) {
    __bf16* drow = p.dq + qhead + row * q_stride;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        bf16x4 w;
#pragma unroll
        for (int t = 0; t < 4; ++t) w[t] = (__bf16)(acc[db][4 * q4 + t] * p.scale);
        *reinterpret_cast<bf16x4*>(drow + 32 * db + 8 * q4 + 4 * h) = w;
      }
  }
}

// ---- dK, dV ------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kThreads, 1) void attn_bwd_dkdv_kernel(AttnParams p) {
  constexpr int BK = 128;  // keys per workgroup, 32 per wavefront
  constexpr int BQ = 64;   // query rows per loop step
  constexpr int NKS = D / 16, NDB = D / 32;
  constexpr int TILE_BYTES = BQ * D * 2;
  constexpr int STAGE_BYTES = 2 * TILE_BYTES + 2 * BQ * 4;  // Q, dO, lse*log2e, delta
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ int scratch[8];

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int n = lane & 31, h = lane >> 5, grp = lane >> 4;

  TileCoord tc = decode_tile<BK>(p, p.Hkv, false, scratch);
  if (!tc.valid) return;
  const int g = tc.h;
  const int group = p.Hq / p.Hkv;
  const int64_t k0 = tc.t0;
  const int64_t q_begin = p.causal ? k0 : tc.doc_begin;
  const int64_t q_end = tc.doc_end;
  const int nqt = (int)((q_end - q_begin + BQ - 1) / BQ);

  const int64_t q_stride = (int64_t)p.Hq * D, kv_stride = (int64_t)p.Hkv * D;
  const int64_t kvhead = ((int64_t)tc.b * p.S * p.Hkv + g) * D;

  // This lane's key (column of S); clamped copies are computed but never written.
  int64_t key = k0 + wv * 32 + n;
  const bool key_ok = key < tc.doc_end;
  const int64_t key_ld = key_ok ? key : tc.doc_end - 1;
  bf16x8 kf[NKS], vf[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    kf[ks] = *reinterpret_cast<const bf16x8*>(p.k + kvhead + key_ld * kv_stride + ks * 16 + h * 8);
    vf[ks] = *reinterpret_cast<const bf16x8*>(p.v + kvhead + key_ld * kv_stride + ks * 16 + h * 8);
  }

  int nat_off[2][NKS];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) nat_off[rb][ks] = tile_off<D>(32 * rb + n, 2 * ks + h);
  int tr0[NDB], tr8[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    tr0[db] = tr_off<D>(lane, 4 * (grp >> 1), 32 * db + 16 * (grp & 1));
    tr8[db] = tr_off<D>(lane, 8 + 4 * (grp >> 1), 32 * db + 16 * (grp & 1));
  }

  f32x16 dkacc[NDB], dvacc[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dkacc[db][r] = 0.f; dvacc[db][r] = 0.f; }

  const float c = p.scale_log2;
  const int total = nqt * group;  // loop steps: query heads of the group x query tiles

  TileRegs<BQ, D> qr, dor;
  float stat_reg = 0.f;  // threads 0..63: lse * log2e of row tid; threads 64..127: delta of row tid-64

  auto load_step = [&](int step) {
    const int hq = g * group + step / nqt;
    const int64_t i0 = q_begin + (int64_t)(step % nqt) * BQ;
    const int64_t qhead = ((int64_t)tc.b * p.S * p.Hq + hq) * D;
    tile_load<BQ, D>(qr, p.q + qhead, q_stride, i0, q_end - 1, tid);
    tile_load<BQ, D>(dor, p.dout + qhead, q_stride, i0, q_end - 1, tid);
    if (tid < 2 * BQ) {
      int64_t i = i0 + (tid & (BQ - 1));
      i = i < q_end ? i : q_end - 1;
      const int64_t idx = ((int64_t)tc.b * p.Hq + hq) * p.S + i;
      stat_reg = tid < BQ ? p.lse[idx] * kLog2e : p.delta[idx];
    }
  };
  auto store_step = [&](char* stage) {
    tile_store<BQ, D>(qr, stage, tid);
    tile_store<BQ, D>(dor, stage + TILE_BYTES, tid);
    if (tid < 2 * BQ) reinterpret_cast<float*>(stage + 2 * TILE_BYTES)[tid] = stat_reg;
  };

  load_step(0);
  store_step(smem);
  __syncthreads();

  for (int step = 0; step < total; ++step) {
    const char* st = smem + (step & 1) * STAGE_BYTES;
    const char* q_lds = st;
    const char* do_lds = st + TILE_BYTES;
    const float* lse_lds = reinterpret_cast<const float*>(st + 2 * TILE_BYTES);
    const float* delta_lds = lse_lds + BQ;
    const bool more = step + 1 < total;
    if (more) load_step(step + 1);

    const int64_t i0 = q_begin + (int64_t)(step % nqt) * BQ;
    // Mask when a key of this wave can exceed a row of the tile (causal) or rows run past the document.
    const bool need_mask = (p.causal && k0 + wv * 32 + 31 > i0) || (i0 + BQ > q_end);

#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) s = mfma32(lds_read8(q_lds, nat_off[rb][ks]), kf[ks], s);
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) dp = mfma32(lds_read8(do_lds, nat_off[rb][ks]), vf[ks], dp);
      if (need_mask) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int64_t i = i0 + 32 * rb + 8 * (r >> 2) + 4 * h + (r & 3);
          if ((p.causal && key > i) || i >= q_end) s[r] = -INFINITY;
        }
      }
      bf16x8 pf[2], dsf[2];
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int ri = 32 * rb + 8 * q4 + 4 * h;
        f32x4 l4 = *reinterpret_cast<const f32x4*>(lse_lds + ri);
        f32x4 d4 = *reinterpret_cast<const f32x4*>(delta_lds + ri);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int r = 4 * q4 + t;
          float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -l4[t]));
          pf[r >> 3][r & 7] = (__bf16)pr;
          dsf[r >> 3][r & 7] = (__bf16)(pr * (dp[r] - d4[t]));
        }
      }
#pragma unroll
      for (int sblk = 0; sblk < 2; ++sblk) {
        const int rowbytes = (32 * rb + 16 * sblk) * (D * 2);
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          bf16x4 lo = lds_read_tr4(do_lds + rowbytes + tr0[db]);
          bf16x4 hi = lds_read_tr4(do_lds + rowbytes + tr8[db]);
          dvacc[db] = mfma32(cat4(lo, hi), pf[sblk], dvacc[db]);
        }
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          bf16x4 lo = lds_read_tr4(q_lds + rowbytes + tr0[db]);
          bf16x4 hi = lds_read_tr4(q_lds + rowbytes + tr8[db]);
          dkacc[db] = mfma32(cat4(lo, hi), dsf[sblk], dkacc[db]);
        }
      }
    }

    if (more) store_step(smem + ((step + 1) & 1) * STAGE_BYTES);
    __syncthreads();
  }

  if (key_ok) {
    __bf16* dkrow = p.dk + kvhead + key * kv_stride;
    __bf16* dvrow = p.dv + kvhead + key * kv_stride;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        bf16x4 wk, wv4;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          wk[t] = (__bf16)(dkacc[db][4 * q4 + t] * p.scale);
          wv4[t] = (__bf16)dvacc[db][4 * q4 + t];
        }
        *reinterpret_cast<bf16x4*>(dkrow + 32 * db + 8 * q4 + 4 * h) = wk;
        *reinterpret_cast<bf16x4*>(dvrow + 32 * db + 8 * q4 + 4 * h) = wv4;
      }
  }
}

template <int D>
static int launch_bwd_d(AttnParams p, int phases, hipStream_t st) {
  hipError_t e;
  if (phases & 1) {  // delta
    constexpr int rows_per_block = (kThreads / (D / 8)) * 8;
    int64_t grid = ceil_div(p.S, rows_per_block) * p.B * p.Hq;
    if (grid >= ((int64_t)1 << 31)) return kErrShape;
    attn_bwd_delta_kernel<D><<<dim3((unsigned)grid), dim3(kThreads), 0, st>>>(p);
    if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e);
  }
  if (phases & 2) {  // dq
    constexpr int smem = 2 * 2 * 64 * D * 2;
    int rc = set_smem(attn_bwd_dq_kernel<D>, smem);
    if (rc) return rc;
    int64_t tiles = tiles_per_head(p.S, 128, p.cu, p.num_docs);
    int64_t grid = tiles * p.B * p.Hq;
    if (grid >= ((int64_t)1 << 31)) return kErrShape;
    p.tiles = (int32_t)tiles;
    attn_bwd_dq_kernel<D><<<dim3((unsigned)grid), dim3(kThreads), smem, st>>>(p);
    if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e);
  }
  if (phases & 4) {  // dk, dv
    constexpr int smem = 2 * (2 * 64 * D * 2 + 2 * 64 * 4);
    int rc = set_smem(attn_bwd_dkdv_kernel<D>, smem);
    if (rc) return rc;
    int64_t tiles = tiles_per_head(p.S, 128, p.cu, p.num_docs);
    int64_t grid = tiles * p.B * p.Hkv;
    if (grid >= ((int64_t)1 << 31)) return kErrShape;
    p.tiles = (int32_t)tiles;
    attn_bwd_dkdv_kernel<D><<<dim3((unsigned)grid), dim3(kThreads), smem, st>>>(p);
    if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e);
  }
  return 0;
}

int launch_bwd(AttnParams p, int D, int phases, hipStream_t st) {
  return D == 64 ? launch_bwd_d<64>(p, phases, st) : launch_bwd_d<128>(p, phases, st);
}

}  // namespace ie
