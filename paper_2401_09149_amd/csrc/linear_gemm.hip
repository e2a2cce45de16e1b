// Linear modules without bias, forward and backward (include/ie_linear.h; Sec. 2.1; Sec. 4.2
// "Computation Profiler": the input of dimension (b, S/s_sp, H) applied to a Linear module):
//   y = x w^T,   dx = dy w,   dw = dy^T x        x [M,K], w [N,K], y, dy [M,N], all bf16 row-major.
// All three are C[I,J] = sum_r A(i,r) B(j,r) with each operand stored either with r contiguous
// ("direct": x and w in the forward, dy in dx) or with its output index contiguous ("transposed":
// w in dx, dy and x in dw), so one kernel template with two flags serves them.
//
// A workgroup of 8 wavefronts (two per SIMD, so that one wave's barrier and LDS waits are
// covered by the other's MFMAs) computes one 256 x 256 tile of C at a time (the grid is one
// workgroup per CU, each walking its share of the tiles); wave (wi, wj) owns 128 x 64 of it as
// 4 x 2 blocks of v_mfma_f32_32x32x16_bf16 (128 accumulator registers).  The contraction runs
// in steps of 64 through two LDS stages of 64 KiB filled by asynchronous global->LDS copies.
// Tiles sit in LDS row-major with swizzled 16-byte chunks; a direct operand's
// fragment is one 16-byte LDS read, a transposed operand's fragment two transpose loads.  The
// products are formed transposed, C^T = B A^T (B's rows as the MFMA's row operand), so that a
// lane ends up holding one row i of C with consecutive j in its registers and the epilogue
// writes 16 bytes per lane.  Each k-step reads 4 + 2 fragments for 8 MFMAs: 0.75 KiB of LDS
// reads per MFMA, plus 0.25 KiB of copy writes.  (Four waves
// owning 128 x 128 each, 0.5 KiB of reads per MFMA, were tried both compiler-scheduled and with
// a hand-written instruction order and a mid-stage barrier: with one wave per SIMD the barrier
// and the issue cost of the copy instructions are exposed, and neither version was faster.)
#include "../../include/ie_linear.h"

#include <hip/hip_runtime.h>

#include "attn_common.hpp"
#include "launch.hpp"

namespace ie {
namespace {

constexpr int kWaves = 8;
constexpr int TI = 256, TJ = 256, TR = 64;
constexpr int G_TILE_BYTES = TI * TR * 2;          // 32 KiB, either layout
constexpr int G_STAGE_BYTES = 2 * G_TILE_BYTES;    // A tile | B tile
constexpr int G_SMEM_BYTES = 2 * G_STAGE_BYTES;
constexpr int kPanel = 8;                          // i-tiles that share a j-tile back to back

struct GemmParams {
  const char* a;   // the operand indexed by (i, r)
  const char* b;   // the operand indexed by (j, r)
  __bf16* c;       // [I][J]
  int64_t I, J, R;
  int64_t a_pitch, b_pitch;  // bytes between rows of a / b as stored
  int64_t c_pitch;           // elements
  int tiles_i, tiles_j, tiles;
};

// Swizzle of a direct tile (256 rows of 128 bytes): the 16-byte chunk c of row r sits at chunk position
// c ^ dswz(r).  A 16-byte LDS read is served 16 lanes at a time across 256 bytes of banks, i.e. two rows
// of this tile side by side, so the 16 consecutive rows of a fragment read must put the requested
// chunk at 8 different positions for the even rows and 8 for the odd ones.  (The attention tiles'
// swizzle, made for 256-byte rows and for transpose loads as well, gives only 4: measured, half of all
// LDS cycles of the forward product were bank conflicts with it.)
__device__ __forceinline__ uint32_t dswz(uint32_t r) { return (r >> 1) & 7u; }

// Asynchronous copy of one operand tile into LDS.  `valid` = rows (direct) or 16-byte chunks
// (transposed) of the tile that exist along the output index; lanes past it repeat the last one.
// WAVES: how many of the workgroup's waves take part in a copy (8: all; 4: waves 0-3 or waves 4-7, see the kernel).
template <bool T, int WAVES>
struct TileCopy {
  static constexpr int NI = 32 / WAVES;   // 1 KiB instructions per wave per tile
  uint32_t row;    // tile row this lane fetches in instruction 0: direct tiles add 8*WAVES per instruction, transposed 2*WAVES
  uint32_t chunk;  // its 16-byte chunk POSITION inside the row
  int wave;
  __device__ __forceinline__ void init(int tid) {
    const int lane = tid & 63;
    wave = __builtin_amdgcn_readfirstlane(tid >> 6) % WAVES;
    row = T ? 2 * wave + lane / 32 : 8 * wave + lane / 8;
    chunk = T ? lane % 32 : lane % 8;
  }
  // `g`: first byte of the tile in global memory (wave-uniform); `lds`: byte address of the tile.
  __device__ __forceinline__ void issue(uint32_t lds, const char* g, uint32_t pitch, int valid) const {
#pragma unroll
    for (int t = 0; t < NI; ++t) {
      uint32_t voff;
      if (!T) {
        const uint32_t r = row + 8 * WAVES * t;
        const uint32_t lc = chunk ^ dswz(r);             // the logical chunk that belongs at this position
        const uint32_t rc = r < (uint32_t)valid ? r : (uint32_t)valid - 1;
        voff = rc * pitch + (lc << 4);
      } else {
        const uint32_t r = row + 2 * WAVES * t;
        const uint32_t lc = chunk ^ swz<256>(r);
        const uint32_t ch = lc < (uint32_t)valid ? lc : (uint32_t)valid - 1;
        voff = r * pitch + (ch << 4);
      }
      async_copy16(voff, g, lds + (uint32_t)(wave + WAVES * t) * 1024);
    }
  }
};

// Fragment of the 32 output indices o .. o+31 of a tile for contraction step ks (16 values of r).
template <bool T>
__device__ __forceinline__ bf16x8 frag(const char* tile, int lane, int o, int ks) {
  const int n = lane & 31, h = lane >> 5;
  if (!T) return lds_read8(tile, (o + n) * 128 + (((2 * ks + h) ^ (int)dswz((uint32_t)(o + n))) << 4));
  const int c0 = o + 16 * ((lane >> 4) & 1), r0 = 16 * ks + 8 * h;
  return cat4(lds_read_tr4(tile + tr_off<256>(lane, r0, c0)), lds_read_tr4(tile + tr_off<256>(lane, r0 + 4, c0)));
}

// One lane's share of a 32 x 32 accumulator block: row i of C, 32 consecutive j, of which the
// first `cols` (a multiple of 8) exist.  Same exchange as store_block32_bf16.
__device__ __forceinline__ void store_block(__bf16* dst, const f32x16& acc, int h, bool ok, int cols) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  uint32_t w[4][2];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      bf16x2_t pr;
      pr[0] = (__bf16)acc[4 * q + 2 * j];
      pr[1] = (__bf16)acc[4 * q + 2 * j + 1];
      w[q][j] = __builtin_bit_cast(uint32_t, pr);
    }
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    uint32_t lo[2], hi[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      auto r = __builtin_amdgcn_permlane32_swap(w[2 * g][j], w[2 * g + 1][j], false, false);
      lo[j] = r[0];
      hi[j] = r[1];
    }
    u32x4 out = {lo[0], lo[1], hi[0], hi[1]};
    if (ok && 16 * g + 8 * h < cols) *reinterpret_cast<u32x4*>(dst + 16 * g + 8 * h) = out;
  }
}

// Tile sequence.  The hardware deals consecutive workgroups round-robin to the 8 XCDs; XCD x
// (= workgroup index % 8) works through a contiguous eighth of the sequence, and the sequence
// walks panels of 8 i-tiles, all 8 against one j-tile before the next j-tile, so that the
// workgroups that run together on an XCD share a few A and B panels in its L2.  `l` numbers the
// tiles of one XCD's eighth.
struct GemmTile {
  const char* ga;  // first byte of the A tile of contraction step 0
  const char* gb;
  int64_t i0, j0;
  int i_valid, j_valid, a_valid, b_valid;
  bool valid;
};
template <bool A_T, bool B_T>
__device__ __forceinline__ GemmTile decode_gemm_tile(const GemmParams& p, int l) {
  GemmTile g;
  const int per = (p.tiles + 7) / 8;
  const int t = (int)(blockIdx.x & 7) * per + l;
  g.valid = l < per && t < p.tiles;
  if (!g.valid) return g;
  const int panel_tiles = kPanel * p.tiles_j;
  const int panel = t / panel_tiles, in_panel = t % panel_tiles;
  const int rows_in_panel = p.tiles_i - panel * kPanel < kPanel ? p.tiles_i - panel * kPanel : kPanel;
  const int tj = in_panel / rows_in_panel;
  const int ti = panel * kPanel + in_panel % rows_in_panel;
  g.i0 = (int64_t)ti * TI;
  g.j0 = (int64_t)tj * TJ;
  g.i_valid = (int)(p.I - g.i0 < TI ? p.I - g.i0 : TI);
  g.j_valid = (int)(p.J - g.j0 < TJ ? p.J - g.j0 : TJ);
  g.ga = p.a + (A_T ? g.i0 * 2 : g.i0 * p.a_pitch);
  g.gb = p.b + (B_T ? g.j0 * 2 : g.j0 * p.b_pitch);
  g.a_valid = A_T ? g.i_valid / 8 : g.i_valid;
  g.b_valid = B_T ? g.j_valid / 8 : g.j_valid;
  return g;
}

template <bool A_T, bool B_T>
__global__ __launch_bounds__(kWaves * 64, 1) void linear_gemm_kernel(GemmParams p) {
  constexpr int NJB = 2;   // 32-column blocks per wave: it owns 128 x 64 of the tile
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int n = lane & 31, h = lane >> 5;
  // Persistent: this workgroup takes every (gridDim/8)-th tile of its XCD's share.  The first
  // copy of the next tile is issued in the last contraction step of the current one, so the
  // epilogue's stores overlap it; the stage parity simply keeps running across tiles.
  int l = (int)(blockIdx.x >> 3);
  const int lstep = (int)(gridDim.x >> 3);
  GemmTile cur = decode_gemm_tile<A_T, B_T>(p, l);
  if (!cur.valid) return;
  const int64_t a_step = A_T ? TR * p.a_pitch : TR * 2;
  const int64_t b_step = B_T ? TR * p.b_pitch : TR * 2;

  // With both operands direct (the forward product) the two waves of a SIMD (w and w + 4) take turns copying: one
  // issues all 16 copy instructions of a stage while the other already has the matrix pipeline, instead of both
  // issuing 8 in front of their first MFMAs (forward products +2-4 %; with a transposed operand the same
  // arrangement loses 2-8 %, so those keep all eight waves copying).
  constexpr bool kTakeTurns = !A_T && !B_T;
  constexpr int kCopyWaves = kTakeTurns ? 4 : kWaves;
  TileCopy<A_T, kCopyWaves> ca;
  TileCopy<B_T, kCopyWaves> cb;
  ca.init(tid);
  cb.init(tid);
  const uint32_t lds0 = lds_address(smem);
  auto copy_stage = [&](const GemmTile& g, int kt, int stage) __attribute__((always_inline)) {
    if (kTakeTurns && (wv >> 2) != (stage & 1)) return;
    const uint32_t base = lds0 + stage * G_STAGE_BYTES;
    ca.issue(base, g.ga + kt * a_step, (uint32_t)p.a_pitch, g.a_valid);
    cb.issue(base + G_TILE_BYTES, g.gb + kt * b_step, (uint32_t)p.b_pitch, g.b_valid);
  };

  const int wi = wv & 1, wj = wv >> 1;   // this wave's part of the tile
  f32x16 acc[4][NJB];
  const int nkt = (int)(p.R / TR);
  int stage = 0;
  copy_stage(cur, 0, 0);
  for (;;) {
    l += lstep;
    const GemmTile nxt = decode_gemm_tile<A_T, B_T>(p, l);
#pragma unroll
    for (int ib = 0; ib < 4; ++ib)
#pragma unroll
      for (int jb = 0; jb < NJB; ++jb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[ib][jb][r] = 0.0f;
    for (int kt = 0; kt < nkt; ++kt) {
      async_wait_all();  // this wave's copies of this stage have landed ...
      __syncthreads();   // ... everyone's have, and everyone is done reading the other stage
      if (kt + 1 < nkt) copy_stage(cur, kt + 1, stage ^ 1);
      else if (nxt.valid) copy_stage(nxt, 0, stage ^ 1);
      const char* ta = smem + stage * G_STAGE_BYTES;
      const char* tb = ta + G_TILE_BYTES;
#pragma unroll
      for (int ks = 0; ks < TR / 16; ++ks) {
        bf16x8 fi[4], fj[NJB];
#pragma unroll
        for (int ib = 0; ib < 4; ++ib) fi[ib] = frag<A_T>(ta, lane, wi * 128 + ib * 32, ks);
#pragma unroll
        for (int jb = 0; jb < NJB; ++jb) fj[jb] = frag<B_T>(tb, lane, wj * (32 * NJB) + jb * 32, ks);
#pragma unroll
        for (int ib = 0; ib < 4; ++ib)
#pragma unroll
          for (int jb = 0; jb < NJB; ++jb) acc[ib][jb] = mfma32(fj[jb], fi[ib], acc[ib][jb]);
      }
      stage ^= 1;
    }
#pragma unroll
    for (int ib = 0; ib < 4; ++ib) {
      const int il = wi * 128 + ib * 32 + n;
      const bool ok = il < cur.i_valid;
      __bf16* crow = p.c + (cur.i0 + (ok ? il : 0)) * p.c_pitch + cur.j0;
#pragma unroll
      for (int jb = 0; jb < NJB; ++jb) {
        const int jl = wj * (32 * NJB) + jb * 32;
        store_block(crow + jl, acc[ib][jb], h, ok, cur.j_valid - jl);
      }
    }
    if (!nxt.valid) break;
    cur = nxt;
  }
}

constexpr int64_t kMaxDim = (int64_t)1 << 22;   // rows stay below 8 MiB: 256 rows of byte offsets fit 32 bits

bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; }

int check_dims(int64_t M, int64_t N, int64_t K) {
  if (M <= 0 || N <= 0 || K <= 0) return IE_ERR_SHAPE;
  if (M >= kMaxDim * 64 || N >= kMaxDim || K >= kMaxDim) return IE_ERR_SHAPE;
  return IE_OK;
}

template <bool A_T, bool B_T>
int launch_gemm(GemmParams p, hipStream_t st) {
  auto kernel = linear_gemm_kernel<A_T, B_T>;
  int rc = set_smem(kernel, G_SMEM_BYTES);
  if (rc) return rc;
  p.tiles_i = (int)ceil_div(p.I, TI);
  p.tiles_j = (int)ceil_div(p.J, TJ);
  const int64_t tiles = (int64_t)p.tiles_i * p.tiles_j;
  if (tiles >= ((int64_t)1 << 28)) return IE_ERR_SHAPE;
  p.tiles = (int)tiles;
  hipError_t e;
  const int cus = cu_count(&e);
  if (e != hipSuccess) return hip_fail(e);
  const int per = (p.tiles + 7) / 8;                      // tiles of one XCD's share
  const int per_xcd_wgs = cus / 8 < per ? cus / 8 : per;  // one workgroup per CU (128 KiB of LDS each)
  const unsigned grid = 8u * (unsigned)(per_xcd_wgs < 1 ? 1 : per_xcd_wgs);
  kernel<<<dim3(grid), dim3(kWaves * 64), G_SMEM_BYTES, st>>>(p);
  e = hipGetLastError();
  return e == hipSuccess ? IE_OK : hip_fail(e);
}

}  // namespace
}  // namespace ie

extern "C" {

int ie_linear_fwd(const void* x, const void* w, void* y, int64_t M, int64_t N, int64_t K, void* stream) {
  if (!x || !w || !y) return IE_ERR_NULL;
  if (int rc = ie::check_dims(M, N, K)) return rc;
  if (K % 64 != 0 || N % 8 != 0) return IE_ERR_UNSUPPORTED;   // contraction over K; rows of y are written 16 bytes at a time
  if (!ie::aligned16(x) || !ie::aligned16(w) || !ie::aligned16(y)) return IE_ERR_ALIGN;
  ie::GemmParams p{};
  p.a = static_cast<const char*>(x); p.b = static_cast<const char*>(w); p.c = static_cast<__bf16*>(y);
  p.I = M; p.J = N; p.R = K;
  p.a_pitch = K * 2; p.b_pitch = K * 2; p.c_pitch = N;
  return ie::launch_gemm<false, false>(p, static_cast<hipStream_t>(stream));
}

int ie_linear_bwd_input(const void* dy, const void* w, void* dx, int64_t M, int64_t N, int64_t K, void* stream) {
  if (!dy || !w || !dx) return IE_ERR_NULL;
  if (int rc = ie::check_dims(M, N, K)) return rc;
  if (N % 64 != 0 || K % 8 != 0) return IE_ERR_UNSUPPORTED;   // contraction over N
  if (!ie::aligned16(dy) || !ie::aligned16(w) || !ie::aligned16(dx)) return IE_ERR_ALIGN;
  ie::GemmParams p{};
  p.a = static_cast<const char*>(dy); p.b = static_cast<const char*>(w); p.c = static_cast<__bf16*>(dx);
  p.I = M; p.J = K; p.R = N;
  p.a_pitch = N * 2; p.b_pitch = K * 2; p.c_pitch = K;
  return ie::launch_gemm<false, true>(p, static_cast<hipStream_t>(stream));
}

int ie_linear_bwd_weight(const void* dy, const void* x, void* dw, int64_t M, int64_t N, int64_t K, void* stream) {
  if (!dy || !x || !dw) return IE_ERR_NULL;
  if (int rc = ie::check_dims(M, N, K)) return rc;
  if (M % 64 != 0 || N % 8 != 0 || K % 8 != 0) return IE_ERR_UNSUPPORTED;   // contraction over M
  if (!ie::aligned16(dy) || !ie::aligned16(x) || !ie::aligned16(dw)) return IE_ERR_ALIGN;
  ie::GemmParams p{};
  p.a = static_cast<const char*>(dy); p.b = static_cast<const char*>(x); p.c = static_cast<__bf16*>(dw);
  p.I = N; p.J = K; p.R = M;
  p.a_pitch = N * 2; p.b_pitch = K * 2; p.c_pitch = K;
  return ie::launch_gemm<true, true>(p, static_cast<hipStream_t>(stream));
}

}  // extern "C"
