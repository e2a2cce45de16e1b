// Forward kernel for head dimension 128, one wave per SIMD: O = softmax(scale * Q K^T + mask) V
// and the per-row log-sum-exp (fused attention of Sec. 2.1 / Sec. 4.2, recast for CDNA4).
//
// One item per (batch, head, 256-query tile), taken by persistent workgroups from a queue
// (tile_queue.hpp); each of the 4 wavefronts owns 64 query rows
// as two 32-row column blocks "a" and "b", whose Q fragments and O^T accumulators stay in
// AGPRs for the whole kernel.  128-key K and V tiles stream through two LDS stages filled by
// asynchronous copies.  Scores are produced transposed, S^T = K Q^T (one query column per
// lane, see attn_fwd.hip), and every K and V^T fragment read from LDS feeds two MFMAs, one per
// column block.
//
// Unmasked tiles run a hand-sequenced pipeline (mfma_asm.hpp).  The softmax of a 32x32 block is
// about 57 VALU instructions against 16 MFMAs, more than fits in the MFMAs' shadow if the two
// are not interleaved instruction by instruction, so the two column blocks are staggered by
// half a block and each phase pairs the MFMAs of one with the softmax of the other
// (i = 32-key block index):
//   A_i: S_a(i+1)_k, PV_a(i)_k alternating, k = 0..7  + softmax of s_b(i)    reads V^T(i+1)
//   B_i: S_b(i+1)_k, PV_b(i)_k alternating            + softmax of s_a(i+1)  reads K(i+2)
// K(i) is read during B_(i-2) and V^T(i) during A_(i-1), so the four blocks of tile T are read
// during the eight phases B_(4T-2) .. A_(4T+2): that is one "round", and the workgroup barrier
// that publishes the next stage and releases this one sits between A_(4T+2) and B_(4T+2).  The
// pipeline never drains at a tile boundary; it is filled in a wave's first round and drained
// after its last unmasked tile.  Tiles that need a mask for this wave (the diagonal, the end of
// a document) take a compiler-scheduled path afterwards.
#include <mutex>
#include <type_traits>

#include "attn_common.hpp"
#include "launch.hpp"
#include "mfma_asm.hpp"
#include "tile_queue.hpp"

namespace ie {

struct FwdWideCfg {
  static constexpr int D = 128;
  static constexpr int BM = 256;                       // query rows per workgroup
  static constexpr int BN = 128;                       // keys per stage
  static constexpr int NB = BN / 32;                   // 32-key blocks per stage
  static constexpr int ROW_BYTES = D * 2;
  static constexpr int PART_BYTES = 64 * ROW_BYTES;    // the asynchronous copy works on 64-row parts
  static constexpr int TILE_BYTES = BN * ROW_BYTES;    // one K or V tile
  static constexpr int V_BASE = 2 * TILE_BYTES;        // LDS: K stage 0 | K stage 1 | V stage 0 | V stage 1
  static constexpr int SMEM_BYTES = 4 * TILE_BYTES;
};

// Softmax state of one 32-query column block (one query per lane, both half-waves alike).
struct ColState {
  float m;      // reference maximum, raw score units (lazy: moves only when exceeded by kSlack)
  float negmc;  // -m * scale * log2(e)
  float thr;    // m + slack
  float l;      // this lane's share of the row sum
};

// CHUNKED: q, k, v are the chunks of a sequence-parallel exchange buffer (tok_off in attn_common.hpp) instead of
// contiguous tensors; a separate instantiation, because this kernel has no register to spare for the general form.
template <bool CHUNKED>
__global__ __launch_bounds__(kThreads, 1) void attn_fwd_wide_kernel(AttnParams p) {
  using C = FwdWideCfg;
  constexpr int D = C::D, BM = C::BM, BN = C::BN, NB = C::NB;
  constexpr int NKS = D / 16, NDB = D / 32;
  constexpr int ROW_BYTES = C::ROW_BYTES, TILE_BYTES = C::TILE_BYTES, V_BASE = C::V_BASE;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ int scratch[8];

  __shared__ QueueState s_work;
  queue_init(p, &s_work);
  const uint32_t xcc = xcc_id();
  int skip = 0;
  for (;;) {   // persistent: one item (batch, head, query tile) per iteration
  const int item = next_work(p, &s_work, xcc, skip);
  if (item < 0) break;
  // Everything below is derived from an opaque copy of the thread index, so that the compiler
  // recomputes the per-lane offsets for every item instead of hoisting them out of this loop and
  // keeping them in registers through the main loop, which has none to spare.
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wv = tid >> 6;
  const int n = lane & 31, h = lane >> 5, grp = lane >> 4;
  TileCoord tc = decode_tile<BM>(p, p.Hq, true, scratch, item, tid);
  if (!tc.valid) continue;
  const int g = tc.h / (p.Hq / p.Hkv);
  const int64_t q0 = tc.t0;
  const int64_t q_end = (q0 + BM < tc.doc_end) ? q0 + BM : tc.doc_end;
  const int64_t k_begin = tc.doc_begin;
  const int64_t k_end = p.causal ? q_end : tc.doc_end;
  // (the tile coordinates may have come through LDS: tell the compiler they are wave-uniform)
  const int nk = (int)uniform((uint32_t)(k_end - k_begin));  // visible keys of the tile (before the per-row causal cut)
  const int nkt = (nk + BN - 1) / BN;

  const int64_t q_stride = (int64_t)p.Hq * D;
  const int64_t kv_pitch = (int64_t)p.Hkv * D * 2;
  // Head tc.h (g) of the batch entry's first token (CHUNKED) or of token k_begin (contiguous tensors); key tile T
  // starts at token k_begin + T * BN.
  const char* qbase = CHUNKED ? reinterpret_cast<const char*>(p.q + tc.h * D) + tc.b * p.q_bstride
                              : reinterpret_cast<const char*>(p.q + ((int64_t)tc.b * p.S * p.Hq + tc.h) * D);
  const char* kbase = uniform(CHUNKED ? reinterpret_cast<const char*>(p.k + g * D) + tc.b * p.kv_bstride
                                      : reinterpret_cast<const char*>(p.k + (((int64_t)tc.b * p.S + k_begin) * p.Hkv + g) * D));
  const char* vbase = uniform(CHUNKED ? reinterpret_cast<const char*>(p.v + g * D) + tc.b * p.kv_bstride
                                      : reinterpret_cast<const char*>(p.v + (((int64_t)tc.b * p.S + k_begin) * p.Hkv + g) * D));
  const int64_t tile_pitch = BN * kv_pitch;
  auto key_tile_off = [&](const int T) __attribute__((always_inline)) {
    if constexpr (CHUNKED) return tok_off(p, k_begin + (int64_t)T * BN, kv_pitch);
    else return T * tile_pitch;
  };
  auto q_row_off = [&](const int64_t row) __attribute__((always_inline)) {
    if constexpr (CHUNKED) return tok_off(p, row, q_stride * 2);
    else return row * q_stride * 2;
  };

  const uint32_t lds0 = lds_address(smem);
  AsyncTile<D> ld;
  ld.init(tid, kv_pitch);
  const int wave_u = ld.wave;

  // Asynchronous copy of key tile T into stage T & 1: all at once (any number of valid rows), or
  // piece by piece for a complete tile (16 pieces per wave: 2 tensors x 2 parts x 4 instructions).
  static_assert(2 * (BN / 64) * AsyncTile<D>::NI == 16, "two pieces per phase, eight phases per round");
  auto copy_all = [&](const int T) __attribute__((always_inline)) {
    const int rows = nk - T * BN;  // >= 1
    const uint32_t base = lds0 + (T & 1) * TILE_BYTES;
#pragma unroll
    for (int part = 0; part < BN / 64; ++part) {
      const int first = rows > 64 * part ? 64 * part : rows - 1;  // a part past the end repeats the last row
      const int valid = rows > 64 * part ? rows - 64 * part : 1;
      ld.load(base + part * C::PART_BYTES, kbase + key_tile_off(T) + (int64_t)first * kv_pitch, valid);
      ld.load(base + V_BASE + part * C::PART_BYTES, vbase + key_tile_off(T) + (int64_t)first * kv_pitch, valid);
    }
  };
  // Piece k of a complete tile: instruction i of 64-row part `part` of tensor `tensor`.  The row
  // offset of the instruction sits in a per-lane offset register and the part's in the scalar base,
  // so that a piece costs three instructions (M0, a wait state, the copy).
  uint32_t voff_i[AsyncTile<D>::NI];
#pragma unroll
  for (int i = 0; i < AsyncTile<D>::NI; ++i) voff_i[i] = ld.voff + (uint32_t)(4 * AsyncTile<D>::RPI * i) * ld.pitch;
  struct CopySrc { const char* k[BN / 64]; const char* v[BN / 64]; uint32_t lds; };
  auto copy_src = [&](const int T) __attribute__((always_inline)) {
    CopySrc cs;
#pragma unroll
    for (int part = 0; part < BN / 64; ++part) {
      cs.k[part] = kbase + key_tile_off(T) + (int64_t)(64 * part) * kv_pitch;
      cs.v[part] = vbase + key_tile_off(T) + (int64_t)(64 * part) * kv_pitch;
    }
    cs.lds = lds0 + (T & 1) * TILE_BYTES + wave_u * 1024;
    return cs;
  };
  auto copy_piece = [&](const CopySrc& cs, const int k) __attribute__((always_inline)) {
    constexpr int NI = AsyncTile<D>::NI;
    const int tensor = k / ((BN / 64) * NI), part = (k / NI) % (BN / 64), i = k % NI;
    async_copy16(voff_i[i], tensor ? cs.v[part] : cs.k[part], cs.lds + tensor * V_BASE + part * C::PART_BYTES + i * 4096);
  };
  copy_all(0);

  // This lane's two query rows (clamped into the tile: out-of-range lanes repeat the last row).
  int64_t row_a = q0 + wv * 64 + n, row_b = row_a + 32;
  const bool ok_a = row_a < q_end, ok_b = row_b < q_end;
  if (!ok_a) row_a = q_end - 1;
  if (!ok_b) row_b = q_end - 1;
  const int rel_a = (int)(row_a - k_begin), rel_b = (int)(row_b - k_begin);

  bf16x8 qa[NKS], qb[NKS];  // live in AGPRs: B operand of S^T = K Q^T, column n = query
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    qa[ks] = global_load_to_agpr(qbase + q_row_off(row_a) + (ks * 16 + h * 8) * 2);
    qb[ks] = global_load_to_agpr(qbase + q_row_off(row_b) + (ks * 16 + h * 8) * 2);
  }

  // Per-lane LDS addresses in stage 0; stage, block and half-block offsets are immediates.
  const char* kp[NKS];   // K tile, A operand: row = key n of a block, chunk = 2ks + h
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) kp[ks] = smem + tile_off<D>(n, 2 * ks + h);
  const char* vp0[NDB];  // V tile, transpose loads: rows 4h.. and 8+4h.. of each 16-key group
  const char* vp8[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    vp0[db] = smem + V_BASE + tr_off<D>(lane, 4 * (grp >> 1), 32 * db + 16 * (grp & 1));
    vp8[db] = smem + V_BASE + tr_off<D>(lane, 8 + 4 * (grp >> 1), 32 * db + 16 * (grp & 1));
  }

  const float c = p.scale_log2;
  constexpr float kSlack = 8.0f;  // log2 units, see attn_fwd.hip
  // The hand-sequenced path lets exponentials grow much further before it moves the reference:
  // a block is done again only if one lane's 16 exponentials sum to more than this (or to NaN).
  // Probabilities up to 2^24 against a reference that lags are harmless in fp32 and in bf16 (both
  // keep 8 exponent bits): the final normalisation by l removes the common factor.
  constexpr float kRedo = 16777216.0f;
  const float slack_raw = kSlack / c;
  ColState sa{-INFINITY, INFINITY, -INFINITY, 0.f}, sb{-INFINITY, INFINITY, -INFINITY, 0.f};
  f32x16 oa[NDB], ob[NDB];  // live in AGPRs
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) { oa[db][r] = 0.f; ob[db][r] = 0.f; }

  // The reference maximum of a column block moves: rescale its accumulators.  Rare after the
  // first blocks of a row.  The accumulators are AGPRs that assembly MFMAs write: fenced.
  auto rescale = [&](ColState& st, f32x16 (&o)[NDB], const float mx) __attribute__((always_inline)) {
    mfma_result_fence();
    const float m_new = fmaxf(st.m, mx);
    const float alpha = __builtin_amdgcn_exp2f((st.m - m_new) * c);
    st.m = m_new;
    st.negmc = -m_new * c;
    st.thr = m_new + slack_raw;
    st.l *= alpha;
    // element by element through one VGPR, in assembly: left to the compiler, the multiplications
    // pull the accumulators out of the AGPRs for whole phases
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float tmp;
        asm volatile("v_accvgpr_read_b32 %1, %0\n\tv_mul_f32 %1, %1, %2\n\ts_nop 0\n\tv_accvgpr_write_b32 %0, %1"
                     : "+a"(o[db][r]), "=&v"(tmp)
                     : "v"(alpha));
      }
    mfma_result_fence();
  };

  // ---- pipeline state that crosses phase and round boundaries
  const int wave_row_min = (int)uniform((uint32_t)((int)(q0 - k_begin) + wv * 64));
  bf16x8 kf[NKS];          // K fragments of the block whose scores come next
  bf16x8 vt[2][2][NDB];    // V^T fragments, double-buffered by block parity: [parity][16-key half][db]
  f32x16 s_a, s_b;         // scores of the current block of each column block
  uint32_t pw_a[8], pw_b[8];  // packed probabilities (bf16 pairs) of each column block
  float pr_a[16], pr_b[16];   // exponentials waiting to be summed and packed
  float lsum_a, lsum_b;       // this lane's sum of the current block's exponentials

  // Element e of a block's softmax: its exponential; the block sum takes the previous element and
  // the pack the previous pair, so that neither reads a v_exp_f32 result in the very next instruction.
  auto elem = [&](float (&pr)[16], uint32_t (&pw)[8], const f32x16& s, const ColState& st, float& lsum, const int e)
      __attribute__((always_inline)) {
    if (e < 2) exp_elem(pr[e], s[e], c, st.negmc);
    else if (e == 2) exp_elem_first_sum(pr[2], s[2], c, st.negmc, lsum, pr[0], pr[1], pw[0]);
    else if (e & 1) exp_elem_add(pr[e], s[e], c, st.negmc, lsum, pr[e - 1]);
    else exp_elem_add_pack(pr[e], s[e], c, st.negmc, lsum, pr[e - 1], pw[e / 2 - 1], pr[e - 2]);
  };
  // A block whose exponentials outgrew the reference (or the very first block of a row): find
  // the true column maximum, move the reference there and form the block's probabilities again.
  // Cold: after its first blocks a row practically never comes here.
  auto redo = [&](ColState& st, f32x16 (&o)[NDB], const f32x16& s, uint32_t (&pw)[8], float& lsum) __attribute__((always_inline)) {
    float mx = s[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
    mx = halfwave_max(mx);
    rescale(st, o, mx);
    lsum = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * t], c, st.negmc));
      const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * t + 1], c, st.negmc));
      pw[t] = __builtin_bit_cast(uint32_t, pack_bf16(e0, e1));
      lsum += e0 + e1;
    }
  };

  // One phase: 16 MFMA slots.  X is the column block whose MFMAs run (S of block i+1 on even
  // slots, PV of block i on odd slots), Y the one whose softmax runs (on s_y).  KLOAD / VLOAD: after a
  // K fragment's last use load the next block's (r = local block index in stage STG, or -1);
  // load the next block's V^T into the other buffer.
  auto phase = [&](auto has_s, auto has_pv, auto has_sm, auto has_tail, const bf16x8 (&qx)[NKS], f32x16& s_x,
                   f32x16 (&o_x)[NDB], uint32_t (&pw_x)[8], float (&pr_x)[16], ColState& st_x, f32x16& s_y,
                   f32x16 (&o_y)[NDB], uint32_t (&pw_y)[8], float (&pr_y)[16], float& lsum_y, ColState& st_y, auto vpar_c,
                   auto kload_c, auto vload_c, const bool copying, const CopySrc& cs, auto slot_c)
      __attribute__((always_inline)) {
    constexpr bool HAS_S = decltype(has_s)::value, HAS_PV = decltype(has_pv)::value;
    constexpr bool HAS_SM = decltype(has_sm)::value;
    constexpr int vpar = decltype(vpar_c)::value, kload_off = decltype(kload_c)::value;
    constexpr int vload_off = decltype(vload_c)::value;
    constexpr int copy_slot = decltype(slot_c)::value;
    bf16x8 pf0, pf1;
#pragma unroll
    for (int pos = 0; pos < 16; ++pos) {
      const int k = pos >> 1;
      // all 16 pieces in the first four phases of the round: what is issued late in the round is
      // still in flight at the barrier that ends it
      if (copying && copy_slot < 4 && (pos & 3) == 0) copy_piece(cs, 4 * copy_slot + (pos >> 2));
      // ---- the MFMA of this slot, and the LDS read that can follow it
      if ((pos & 1) == 0) {
        if (HAS_S) {
          if (k == 0) mfma_first_b_agpr(s_x, kf[0], qx[0]);
          else mfma_next_b_agpr(s_x, kf[k], qx[k]);
        }
        if (kload_off >= 0) kf[k] = lds_read8(kp[k], kload_off);
      } else {
        if (HAS_PV) {
          if (k == 0) pf0 = frag_from_words(pw_x[0], pw_x[1], pw_x[2], pw_x[3]);
          if (k == NDB) pf1 = frag_from_words(pw_x[4], pw_x[5], pw_x[6], pw_x[7]);
          mfma_acc_agpr(o_x[k % NDB], vt[vpar][k / NDB][k % NDB], k < NDB ? pf0 : pf1);
        }
        if (vload_off >= 0) {
          const int off = vload_off + 16 * (k / NDB) * ROW_BYTES;
          vt[vpar ^ 1][k / NDB][k % NDB] = cat4(lds_read_tr4(vp0[k % NDB] + off), lds_read_tr4(vp8[k % NDB] + off));
        }
      }
      // ---- the VALU work of this slot: the softmax of s_y.  Its scores were complete four MFMAs
      // before slot 2.  There is no running maximum: the exponentials are taken against the
      // column's current reference, and only a block whose sum shows that the reference is too
      // low (or not set yet) is done again.
      if (HAS_SM) {
        if (pos >= 2 && pos <= 4) { elem(pr_y, pw_y, s_y, st_y, lsum_y, 2 * (pos - 2)); elem(pr_y, pw_y, s_y, st_y, lsum_y, 2 * (pos - 2) + 1); }
        if (pos >= 5 && pos <= 14) elem(pr_y, pw_y, s_y, st_y, lsum_y, pos + 1);
        if (pos == 15) {
          add_pack(lsum_y, pr_y[15], pw_y[7], pr_y[14]);
          if (__builtin_amdgcn_ballot_w64(!(lsum_y <= kRedo)) != 0) redo(st_y, o_y, s_y, pw_y, lsum_y);
          st_y.l += lsum_y;
        }
      }
      asm_fence();
    }
  };
  // shorthands for the two kinds of phase
  using Y = std::true_type;
  using N = std::false_type;
  using None = std::integral_constant<int, -1>;
  bool copying = false;  // the current round copies the next tile piece by piece
  CopySrc cs{};
  auto phase_a = [&](auto has_s, auto has_pv, auto has_sm, auto has_tail, auto vpar, auto vload_off, auto copy_slot)
      __attribute__((always_inline)) {
    phase(has_s, has_pv, has_sm, has_tail, qa, s_a, oa, pw_a, pr_a, sa, s_b, ob, pw_b, pr_b, lsum_b, sb, vpar, None{}, vload_off, copying, cs, copy_slot);
  };
  auto phase_b = [&](auto has_s, auto has_pv, auto has_sm, auto has_tail, auto vpar, auto kload_off, auto copy_slot)
      __attribute__((always_inline)) {
    phase(has_s, has_pv, has_sm, has_tail, qb, s_b, ob, pw_b, pr_b, sb, s_a, oa, pw_a, pr_a, lsum_a, sa, vpar, kload_off, None{}, copying, cs, copy_slot);
  };

  // One round: the eight phases that read tile T (stage STG).  `copy_tile` is T + 1 when that
  // tile is complete and is to be copied piece by piece during the round, else -1.
  auto round = [&](auto stg_c, auto first_c, const int copy_tile) __attribute__((always_inline)) {
    copying = copy_tile >= 0;
    if (copying) cs = copy_src(copy_tile);
    constexpr int STG = decltype(stg_c)::value;
    constexpr bool FIRST = decltype(first_c)::value;
    constexpr int so = STG * TILE_BYTES;
    constexpr int BB = 32 * ROW_BYTES;  // bytes per block
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using O0 = std::integral_constant<int, so>;
    using O1 = std::integral_constant<int, so + BB>;
    using O2 = std::integral_constant<int, so + 2 * BB>;
    using O3 = std::integral_constant<int, so + 3 * BB>;
    if (FIRST) {
      // fill: K(0); S_a(0) with V^T(0); S_b(0) with the softmax of s_a(0) and K(1)
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) kf[ks] = lds_read8(kp[ks], so);
      if (copying) { copy_piece(cs, 0); copy_piece(cs, 1); copy_piece(cs, 2); copy_piece(cs, 3); }  // the pieces of the phase that has no MFMAs
      asm_fence();
      phase_a(Y{}, N{}, N{}, N{}, I1{}, O0{}, I1{});
      phase_b(Y{}, N{}, Y{}, N{}, I1{}, O1{}, std::integral_constant<int, 2>{});
    } else {
      phase_b(Y{}, Y{}, Y{}, Y{}, I0{}, O0{}, I0{});                                  // B(prev 2)
      phase_a(Y{}, Y{}, Y{}, Y{}, I1{}, O0{}, I1{});                                  // A(prev 3)
      phase_b(Y{}, Y{}, Y{}, Y{}, I1{}, O1{}, std::integral_constant<int, 2>{});      // B(prev 3)
    }
    phase_a(Y{}, Y{}, Y{}, Y{}, I0{}, O1{}, std::integral_constant<int, 3>{});        // A(0)
    phase_b(Y{}, Y{}, Y{}, Y{}, I0{}, O2{}, std::integral_constant<int, 4>{});        // B(0)
    phase_a(Y{}, Y{}, Y{}, Y{}, I1{}, O2{}, std::integral_constant<int, 5>{});        // A(1)
    phase_b(Y{}, Y{}, Y{}, Y{}, I1{}, O3{}, std::integral_constant<int, 6>{});        // B(1)
    phase_a(Y{}, Y{}, Y{}, Y{}, I0{}, O3{}, std::integral_constant<int, 7>{});        // A(2)
  };
  // After a wave's last round: finish blocks 2 and 3 of that tile from registers.
  auto drain = [&]() __attribute__((always_inline)) {
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    copying = false;
    phase_b(Y{}, Y{}, Y{}, Y{}, I0{}, None{}, I0{});   // B(2): S_b(3), PV_b(2), softmax of s_a(3)
    phase_a(N{}, Y{}, Y{}, Y{}, I1{}, None{}, I0{});   // A(3): PV_a(3), softmax of s_b(3)
    phase_b(N{}, Y{}, N{}, Y{}, I1{}, None{}, I0{});   // B(3): PV_b(3)
    mfma_result_fence();
  };

  // ---- masked tiles: compiler-scheduled.  Per 32-key block both score chains first, then both
  // masks and maxima (with the rare rescale), then the exponentials and the two PV products in
  // one region, so that the compiler can run one column block's MFMAs under the other's
  // exponentials; the next block's fragments are requested before the current block is worked on.
  // (returns whether the block's maximum lies above the column's reference by more than the slack)
  auto masked_max = [&](f32x16& s, const int lim, const ColState& st, float& mx) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (8 * (r >> 2) + (r & 3) > lim) s[r] = -INFINITY;
    mx = s[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
    mx = halfwave_max(mx);
    return __builtin_amdgcn_ballot_w64(mx > st.thr) != 0;
  };
  auto exps = [&](const f32x16& s, ColState& st, bf16x8 (&pf)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int sblk = 0; sblk < 2; ++sblk) {
      bf16x2 pp[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[8 * sblk + 2 * t], c, st.negmc));
        const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[8 * sblk + 2 * t + 1], c, st.negmc));
        pp[t] = pack_bf16(e0, e1);
        st.l += e0 + e1;
      }
      pf[sblk] = cat_pairs(pp[0], pp[1], pp[2], pp[3]);
    }
  };
  auto pv = [&](f32x16 (&o_x)[NDB], const bf16x8 (&vtf)[2][NDB], const bf16x8 (&pf)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int sblk = 0; sblk < 2; ++sblk)
#pragma unroll
      for (int db = 0; db < NDB; ++db) mfma_acc_agpr_after_moves(o_x[db], vtf[sblk][db], pf[sblk]);
    // (assembly, so that the accumulators stay in AGPRs; the compiler does not know these are MFMAs and may move
    // an accumulator right behind them: their results have to have landed)
    mfma_result_fence();
  };
  // Blocks r_begin.. of tile T; returns NB when done.  The rescale of 64 accumulators per column block is cold code,
  // but with it inside the block loop the compiler copies all 128 accumulators out of the AGPRs at the top of every
  // trip; so the loop exists twice: the `lazy` form has no rescale and leaves at the first block whose reference has
  // to move (returning its index, nothing of that block done), and the other form takes over from there.
  auto generic_blocks = [&](const int T, const int r_begin, auto lazy_c) __attribute__((always_inline)) {
    constexpr bool kLazy = decltype(lazy_c)::value;
    const int so = (T & 1) * TILE_BYTES;
    const int kb = T * BN;
    bf16x8 kfr[NKS], vtf[2][NDB];
    auto load_k = [&](const int r) __attribute__((always_inline)) {
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) kfr[ks] = lds_read8(kp[ks], so + 32 * r * ROW_BYTES);
    };
    auto load_v = [&](const int r) __attribute__((always_inline)) {
#pragma unroll
      for (int sblk = 0; sblk < 2; ++sblk)
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          const int off = so + (32 * r + 16 * sblk) * ROW_BYTES;
          vtf[sblk][db] = cat4(lds_read_tr4(vp0[db] + off), lds_read_tr4(vp8[db] + off));
        }
    };
    // a block is worked on when some row of the wave can see some of its keys
    auto visible = [&](const int r) __attribute__((always_inline)) {
      const int key0 = kb + 32 * r;
      return r < NB && key0 < nk && !(p.causal && key0 > wave_row_min + 63);
    };
    if (visible(r_begin)) { load_k(r_begin); load_v(r_begin); }
    int r = r_begin;
#pragma unroll 1
    for (; r < NB; ++r) {
      if (!visible(r)) return NB;
      const bool more = visible(r + 1);
      const int key0 = kb + 32 * r;  // first key of the block, relative to k_begin
      // last visible key relative to the lane's first key of the block (keys 4h.. of each 8)
      const int lim_a = (p.causal ? rel_a : nk - 1) - key0 - 4 * h;
      const int lim_b = (p.causal ? rel_b : nk - 1) - key0 - 4 * h;
      const bool do_a = !(p.causal && key0 > wave_row_min + 31);  // column a's rows end 32 earlier
      bf16x8 pf_a[2], pf_b[2];
      f32x16 ss_a, ss_b;
      if (do_a) ss_a = mfma_chain_b_in_agpr<NKS>(kfr, qa);
      ss_b = mfma_chain_b_in_agpr<NKS>(kfr, qb);
      if (more) load_k(r + 1);  // the K fragments are free again: the next block's, a block ahead of their use
      float mx_a = 0.f, mx_b = 0.f;
      const bool move_a = do_a && masked_max(ss_a, lim_a, sa, mx_a);
      const bool move_b = masked_max(ss_b, lim_b, sb, mx_b);
      if (kLazy) {
        if (move_a || move_b) return r;
      } else {
        if (move_a) rescale(sa, oa, mx_a);
        if (move_b) rescale(sb, ob, mx_b);
      }
      if (do_a) {
        exps(ss_a, sa, pf_a);
        pv(oa, vtf, pf_a);
      }
      exps(ss_b, sb, pf_b);
      pv(ob, vtf, pf_b);
      if (more) load_v(r + 1);
    }
    return NB;
  };
  auto generic_tile = [&](const int T) __attribute__((always_inline)) {
    const int r = generic_blocks(T, 0, std::true_type{});
    if (r < NB) generic_blocks(T, r, std::false_type{});
  };

  // Leading tiles that need no mask for this wave: complete, and (causal) entirely at or below
  // the wave's first row.
  int n_fast = nk / BN;
  if (p.causal) {
    const int below = (wave_row_min + 1) / BN;
    n_fast = n_fast < below ? n_fast : below;
  }

  // The four waves run the same instruction sequence; released together by the barrier they would
  // reach every copy instruction in the same cycle and queue in the CU's one vector-memory path
  // (about 16 cycles per instruction), holding back the MFMAs behind.  A delay of 20 cycles per
  // wave index after each barrier keeps them apart for the whole round.
  auto stagger = [&]() __attribute__((always_inline)) {
    if (wave_u >= 1) asm volatile("s_nop 15\n\ts_nop 3");
    if (wave_u >= 2) asm volatile("s_nop 15\n\ts_nop 3");
    if (wave_u >= 3) asm volatile("s_nop 15\n\ts_nop 3");
  };
  agpr_loads_wait();  // Q fragments (and the first tile's copies) have arrived
  async_wait_all();
  __syncthreads();
  stagger();

  auto end_of_tile = [&]() __attribute__((always_inline)) {
    async_wait_all();  // this wave's copies of the next tile have landed ...
    __syncthreads();   // ... everyone's have, and everyone is done reading this stage
    stagger();
  };
  // Starts the copy of tile T + 1 unless it is left to the round (a complete tile, piece by
  // piece); returns the tile the round has to copy, or -1.
  auto next_copy = [&](const int T) __attribute__((always_inline)) {
    const bool next_full = (T + 2) * BN <= nk;
    if (!next_full && T + 1 < nkt) copy_all(T + 1);
    return next_full ? T + 1 : -1;
  };
  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;
  int T = 0;
  if (n_fast > 0) {
    round(S0{}, Y{}, next_copy(0));
    end_of_tile();
    // steady state, two rounds per trip so that the stage offsets are compile-time constants
    for (T = 1; T + 1 < n_fast; T += 2) {
      round(S1{}, N{}, next_copy(T));
      end_of_tile();
      round(S0{}, N{}, next_copy(T + 1));
      end_of_tile();
    }
    if (T < n_fast) {
      round(S1{}, N{}, next_copy(T));
      end_of_tile();
      ++T;
    }
    drain();
  }
  for (; T < nkt; ++T) {
    if (T + 1 < nkt) copy_all(T + 1);
    // The barrier publishes the next tile and releases this tile's stage for the tile after the next.  The item's
    // last tile but one has no such successor, so the waves that work on it here pass the barrier first: the waves
    // for which that tile needed no mask (the lower half of a causal query tile) then start on the last tile
    // without waiting for this one, and the two diagonal tiles are worked on side by side.
    const bool barrier_first = T + 2 == nkt;
    if (barrier_first) end_of_tile();
    generic_tile(T);
    if (!barrier_first) end_of_tile();
  }
  mfma_result_fence();

  // Epilogue: normalise, write O (bf16) and LSE (natural log).
  auto store = [&](const f32x16 (&o)[NDB], const ColState& st, const int64_t row, const bool ok) __attribute__((always_inline)) {
    const float l_full = halfwave_sum(st.l);
    const float inv_l = 1.0f / l_full;
    __bf16* orow = p.o_out + ((int64_t)tc.b * p.S * p.Hq + tc.h) * D + row * q_stride;
#pragma unroll
    for (int db = 0; db < NDB; ++db) store_block32_bf16(orow + 32 * db, o[db], inv_l, h, ok);
    if (ok && h == 0) p.lse_out[((int64_t)tc.b * p.Hq + tc.h) * p.S + row] = (st.m * c + __builtin_amdgcn_logf(l_full)) * kLn2;
  };
  // (the rows are formed again from their 32-bit positions: two 64-bit row indices kept alive
  // through the whole kernel are four registers this kernel does not have)
  store(oa, sa, k_begin + rel_a, ok_a);
  store(ob, sb, k_begin + rel_b, ok_b);
  }  // next item
  queue_leave(&s_work);
}

// ---- counter slots of the forward's work queue ------------------------------------------------
// The forward has no workspace argument, so its launches take their eight queue counters from a pool
// of slots in a file-scope device array.  A slot must belong to one launch at a time: the host records
// an event behind every launch and hands a slot out again only when that event has completed, or to a
// launch on the same stream (which runs after it anyway); a slot used under stream capture stays with
// that graph for good (its replays are invisible to the host).  When every slot is in flight on other
// streams or pinned, the call fails with IE_ERR_BUSY instead of sharing one.
constexpr int kFwdSlots = 256;
static __device__ __align__(256) unsigned int g_fwd_queue[kFwdSlots * (kQueueBytes / 4)];

namespace {
enum : unsigned char { kSlotFree = 0, kSlotPending = 1, kSlotPinned = 2, kSlotLaunching = 3 };
struct SlotPool {
  std::mutex mu;
  unsigned int* base = nullptr;       // device address of g_fwd_queue on this device
  hipEvent_t ev[kFwdSlots] = {};      // behind the slot's latest launch (created on first use)
  hipStream_t stream[kFwdSlots] = {}; // the stream of that launch
  unsigned char state[kFwdSlots] = {};
  int next = 0;
};
SlotPool g_pools[kMaxDevices];

// Returns 0 and a slot (index, device address of its counters), or a status.
int slot_acquire(hipStream_t st, int* dev_out, int* slot_out, unsigned int** counters, bool* capturing) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  if (dev >= kMaxDevices) return kErrBusy;
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if ((e = hipStreamIsCapturing(st, &cs)) != hipSuccess) return hip_fail(e);
  *capturing = cs == hipStreamCaptureStatusActive;
  SlotPool& pool = g_pools[dev];
  std::lock_guard<std::mutex> lock(pool.mu);
  if (pool.base == nullptr) {
    void* ptr = nullptr;
    if ((e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_fwd_queue))) != hipSuccess) return hip_fail(e);
    pool.base = static_cast<unsigned int*>(ptr);
  }
  // (querying an event is not allowed while this thread captures in the default mode: relax the mode around it)
  hipStreamCaptureMode mode = hipStreamCaptureModeRelaxed;
  if (*capturing && (e = hipThreadExchangeStreamCaptureMode(&mode)) != hipSuccess) return hip_fail(e);
  int found = -1;
  for (int i = 0; i < kFwdSlots && found < 0; ++i) {
    const int s = (pool.next + i) % kFwdSlots;
    if (pool.state[s] == kSlotPending) {
      const hipError_t q = hipEventQuery(pool.ev[s]);
      if (q == hipSuccess) pool.state[s] = kSlotFree;
      else (void)hipGetLastError();   // "not ready" must not be taken for a launch failure later on
    }
    if (pool.state[s] == kSlotFree) found = s;
  }
  if (*capturing) (void)hipThreadExchangeStreamCaptureMode(&mode);
  // nothing has completed: a slot whose launch sits earlier on this very stream is as good
  for (int i = 0; i < kFwdSlots && found < 0 && !*capturing; ++i) {
    const int s = (pool.next + i) % kFwdSlots;
    if (pool.state[s] == kSlotPending && pool.stream[s] == st) found = s;
  }
  if (found >= 0) {
    pool.state[found] = kSlotLaunching;
    pool.next = (found + 1) % kFwdSlots;
    *dev_out = dev;
    *slot_out = found;
    *counters = pool.base + found * (kQueueBytes / 4);
    return 0;
  }
  return kErrBusy;
}

// After the launch (or a failed attempt): ties the slot to what was enqueued.
void slot_release(int dev, int slot, hipStream_t st, bool capturing, bool launched) {
  SlotPool& pool = g_pools[dev];
  std::lock_guard<std::mutex> lock(pool.mu);
  if (!launched) { pool.state[slot] = kSlotFree; return; }
  if (capturing) { pool.state[slot] = kSlotPinned; return; }
  if (pool.ev[slot] == nullptr && hipEventCreateWithFlags(&pool.ev[slot], hipEventDisableTiming) != hipSuccess) {
    (void)hipGetLastError();
    pool.ev[slot] = nullptr;
    pool.state[slot] = kSlotPinned;   // without an event the slot cannot be shown to be free again
    return;
  }
  if (hipEventRecord(pool.ev[slot], st) != hipSuccess) {
    (void)hipGetLastError();
    pool.state[slot] = kSlotPinned;
    return;
  }
  pool.stream[slot] = st;
  pool.state[slot] = kSlotPending;
}
}  // namespace

int launch_fwd_wide(AttnParams p, hipStream_t st) {
  constexpr int smem = FwdWideCfg::SMEM_BYTES;
  const bool chunked = p.tok_shift < 63;
  static KernelSetup setup[2];
  int per_cu = 1;
  int rc = chunked ? kernel_setup(setup[1], attn_fwd_wide_kernel<true>, smem, &per_cu)
                   : kernel_setup(setup[0], attn_fwd_wide_kernel<false>, smem, &per_cu);
  if (rc) return rc;
  int64_t tiles = tiles_per_head(p.S, FwdWideCfg::BM, p.cu, p.num_docs);
  int64_t items = tiles * p.B * p.Hq;
  if (items >= ((int64_t)1 << 31)) return kErrShape;
  p.tiles = (int32_t)tiles;
  int dev = 0, slot = 0;
  unsigned int* counters = nullptr;
  bool capturing = false;
  if ((rc = slot_acquire(st, &dev, &slot, &counters, &capturing)) != 0) return rc;
  // (the slot's counters are zeros: they start out so, and every launch leaves them so, see queue_leave)
  const QueueLaunch ql = tile_queue_prepare(p, counters, items, p.Hq, 1, st, true);
  if (ql.err != hipSuccess) { slot_release(dev, slot, st, capturing, false); return hip_fail(ql.err); }
  if (chunked) attn_fwd_wide_kernel<true><<<dim3((unsigned)ql.grid), dim3(kThreads), smem, st>>>(p);
  else attn_fwd_wide_kernel<false><<<dim3((unsigned)ql.grid), dim3(kThreads), smem, st>>>(p);
  hipError_t e = hipGetLastError();
  slot_release(dev, slot, st, capturing, e == hipSuccess);   // (a launch that failed has enqueued nothing: the counters are untouched)
  return e == hipSuccess ? 0 : hip_fail(e);
}

}  // namespace ie
