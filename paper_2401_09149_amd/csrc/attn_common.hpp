// Device-side building blocks shared by the gfx950 attention kernels: vector types, the
// MFMA wrappers with their operand layouts, the swizzled LDS tile layout, tile loaders
// and the mapping from a workgroup index to (batch, head, document, tile).
//
// MFMA operand layouts used throughout (wave64, lane l, h = l / 32):
//   v_mfma_f32_32x32x16_bf16  C[m][n] += sum_k A[m][k] * B[k][n]
//     A: lane holds row m = l % 32, k = 8h .. 8h+7           (8 bf16)
//     B: lane holds col n = l % 32, k = 8h .. 8h+7           (8 bf16)
//     C: lane holds col n = l % 32; register r (0..15) is row m = 8 (r / 4) + 4h + r % 4
//   Because C keeps one column per lane and spreads rows over registers, a product
//   whose ROW index is the next contraction index can feed the next MFMA's B operand
//   straight from registers: registers 8s .. 8s+7 of C are rows
//   {16s + 4h + 0..3, 16s + 8 + 4h + 0..3}, which is the k-slot order the A operand of
//   the second product has to follow.
//   ds_read_b64_tr_b16 (LDS transpose load): inside each group of 16 lanes, lane i
//   receives element (i % 4) of the 64-bit words addressed by lanes i/4, 4 + i/4,
//   8 + i/4 and 12 + i/4.  With lane L addressing row r0 + L/4, columns c0 + 4 (L%4)..+3
//   of a row-major tile, lane i gets rows r0 .. r0+3 of column c0 + i: a column gather,
//   which is what an MFMA operand needs when the contraction runs over tile rows.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ie {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;   // 4 wavefronts per workgroup
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct AttnParams {
  const __bf16* q; const __bf16* k; const __bf16* v; const __bf16* o; const __bf16* dout;
  __bf16* o_out; float* lse_out;
  const float* lse; float* delta; float* lse2;  // workspace, written by the delta kernel: -delta and -lse * log2(e)
  __bf16* dq; __bf16* dk; __bf16* dv;
  const int32_t* cu; int32_t num_docs;
  int64_t B, S;
  int32_t Hq, Hkv;
  float scale, scale_log2;  // scale_log2 = scale * log2(e)
  int32_t causal;
  int32_t tiles;            // tiles per head the grid was sized for (upper bound when packed)
  int32_t q_heavy, q_per_xcd, q_total;  // persistent launches (tile_queue.hpp): tiles per head in a list's head-by-head part, items per XCD list (0: one list), items
  __bf16* ds;               // optional workspace: dS written by the dK/dV kernel for the dQ kernel (see ds_matrix_offset), or NULL
  // Where token t of batch entry b lives in q/dq (pitch Hq*D) and k/v/dk/dv (pitch Hkv*D), see tok_off():
  // contiguous [B,S,heads,D] tensors, or the chunks of a sequence-parallel exchange buffer (one chunk per peer).
  int32_t tok_shift;              // log2(tokens per chunk); 63 for contiguous tensors
  int64_t tok_mask;               // tokens per chunk - 1; all ones for contiguous tensors
  int64_t tok_cstride;            // bytes between consecutive chunks of one batch entry
  int64_t q_bstride, kv_bstride;  // bytes between batch entries
  unsigned int* q_counters;       // persistent launches: this launch's eight work-queue counters
  unsigned int* ws_counters;      // backward: counter blocks in the caller's workspace (kQueueBytes each, one per kernel)
};

// Layout of the dS workspace (dense input, S a multiple of 128, head dimension 128): for every
// (batch b, query head hq, 128-query tile it) the elements dS[query][key] of the tile's queries and the keys they
// can see (causal: keys 0 .. 128 (it + 1); otherwise all S), bf16, 256 bytes per key; the blocks of one head follow
// each other by it, heads by (b, hq).
// Inside a block the order is the one in which the dK/dV kernel holds dS in registers, so that a wavefront stores
// 2 KiB contiguous: [32-key group][32-query block rb][half-wave hh][key n of the group, at slot n ^ 4 hh]
// [16 values e], where value e belongs to query 32 rb + 8 (e / 4) + 4 hh + e % 4 (register e of the score
// block's C layout).  The dQ kernel copies 32-key groups (8 KiB) into LDS as they are; the exchange of slots
// n and n ^ 4 for hh = 1 spreads its transpose loads over the banks.
__host__ __device__ inline int64_t ds_matrix_offset(int64_t nt, int64_t bh, int64_t it, bool causal) {   // in bytes
  return causal ? (bh * (nt * (nt + 1) / 2) + it * (it + 1) / 2) * 32768 : (bh * nt + it) * nt * 32768;
}
// Bytes between the blocks of query tiles it and it + 1 of one head.
__host__ __device__ inline int64_t ds_matrix_bytes(int64_t nt, int64_t it, bool causal) { return (causal ? it + 1 : nt) * 32768; }

// Byte offset of token t (0 <= t < S) inside its batch entry, for q, k, v and their gradients; `pitch` = bytes per
// token (heads * D * 2).  Contiguous tensors: t * pitch.  Exchange-buffer chunks of 2^tok_shift tokens: the chunk's
// offset plus the row's.
__device__ __forceinline__ int64_t tok_off(const AttnParams& p, int64_t t, int64_t pitch) {
  return (t >> p.tok_shift) * p.tok_cstride + (t & p.tok_mask) * pitch;
}

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// acc = sum_ks A[ks] * B[ks] with the B fragments held in accumulation registers (AGPRs).
// Kernels that run one wave per SIMD keep their stationary operands there: the register
// file has 256 architectural + 256 accumulation registers per lane, but left to itself the
// compiler parks such operands in AGPRs and copies them back (v_accvgpr_read) in front of
// every MFMA, which costs four VALU slots per MFMA.  Written as one assembly block the MFMAs
// read the AGPRs directly.  The block ends with the wait states an 8-pass MFMA needs before
// a VALU instruction may read its result (the compiler's hazard recogniser does not look
// inside inline assembly).
template <int NKS>
__device__ __forceinline__ f32x16 mfma_chain_b_in_agpr(const bf16x8 (&a)[NKS], const bf16x8 (&b)[NKS]) {
  f32x16 acc;
  static_assert(NKS == 8 || NKS == 4, "head dimension 128 or 64");
  if constexpr (NKS == 8) {
    asm volatile(
        "v_mfma_f32_32x32x16_bf16 %0, %1, %9, 0\n\t"
        "v_mfma_f32_32x32x16_bf16 %0, %2, %10, %0\n\t"
        "v_mfma_f32_32x32x16_bf16 %0, %3, %11, %0\n\t"
        "v_mfma_f32_32x32x16_bf16 %0, %4, %12, %0\n\t"
        "v_mfma_f32_32x32x16_bf16 %0, %5, %13, %0\n\t"
        "v_mfma_f32_32x32x16_bf16 %0, %6, %14, %0\n\t"
        "v_mfma_f32_32x32x16_bf16 %0, %7, %15, %0\n\t"
        "v_mfma_f32_32x32x16_bf16 %0, %8, %16, %0\n\t"
        "s_nop 15"
        : "=&v"(acc)
        : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]),
          "a"(b[0]), "a"(b[1]), "a"(b[2]), "a"(b[3]), "a"(b[4]), "a"(b[5]), "a"(b[6]), "a"(b[7]));
  } else {
    asm volatile(
        "v_mfma_f32_32x32x16_bf16 %0, %1, %5, 0\n\t"
        "v_mfma_f32_32x32x16_bf16 %0, %2, %6, %0\n\t"
        "v_mfma_f32_32x32x16_bf16 %0, %3, %7, %0\n\t"
        "v_mfma_f32_32x32x16_bf16 %0, %4, %8, %0\n\t"
        "s_nop 15"
        : "=&v"(acc)
        : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "a"(b[0]), "a"(b[1]), "a"(b[2]), "a"(b[3]));
  }
  return acc;
}

// 16-byte global load straight into accumulation registers (for operands that stay there
// for the whole kernel).  The compiler does not know this is a load: call agpr_loads_wait()
// before the first use.
__device__ __forceinline__ bf16x8 global_load_to_agpr(const void* ptr) {
  bf16x8 r;
  asm volatile("global_load_dwordx4 %0, %1, off" : "=a"(r) : "v"(ptr) : "memory");
  return r;
}
// The same from LDS (byte address `lds_addr`, 16-byte aligned).
__device__ __forceinline__ bf16x8 lds_load_to_agpr(uint32_t lds_addr) {
  bf16x8 r;
  asm volatile("ds_read_b128 %0, %1" : "=a"(r) : "v"(lds_addr) : "memory");
  return r;
}
// A fragment computed in VGPRs, moved into accumulation registers through a lane-private
// 16-byte LDS slot (`lds_addr`, 16-byte aligned): there is no 128-bit VGPR->AGPR move, and a
// value the compiler itself holds is copied over again before every assembly use.  A wave's
// LDS operations complete in order, so the read returns what the write stored.  As above,
// call agpr_loads_wait() before the first use.
__device__ __forceinline__ bf16x8 move_to_agpr_via_lds(bf16x8 x, uint32_t lds_addr) {
  bf16x8 r;
  asm volatile("ds_write_b128 %1, %2\n\tds_read_b128 %0, %1" : "=a"(r) : "v"(lds_addr), "v"(x) : "memory");
  return r;
}
__device__ __forceinline__ void agpr_loads_wait() { asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory"); }

// Exchange between the two half-waves with v_permlane32_swap: given (a, b) it returns
// r0 = {a[0..31], b[0..31]} and r1 = {a[32..63], b[32..63]}.  With a == b == x, lane l
// sees x[l] and x[l ^ 32] in (r0, r1) (in some order).  The vector elements are copied to
// scalars before the bit cast: a bit cast applied to `r[1]` directly reads element 0.
__device__ __forceinline__ void halfwave_pair(float x, float& r0, float& r1) {
  const uint32_t a = __builtin_bit_cast(uint32_t, x);
  auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
  const uint32_t u0 = r[0], u1 = r[1];
  r0 = __builtin_bit_cast(float, u0);
  r1 = __builtin_bit_cast(float, u1);
}
// Maximum / sum over the two half-waves: lane l and lane l ^ 32 both end up with the result.
__device__ __forceinline__ float halfwave_max(float x) {
  float r0, r1;
  halfwave_pair(x, r0, r1);
  return fmaxf(r0, r1);
}
__device__ __forceinline__ float halfwave_sum(float x) {
  float r0, r1;
  halfwave_pair(x, r0, r1);
  return r0 + r1;
}

// Writes one lane's share of a 32-row block of a C-layout accumulator column (16 values: register
// 4 q + t is row 8 q + 4 h + t of the block) as bf16 to the 32 contiguous elements `dst`, scaled by
// `mul`, if `ok`.  The two half-waves first exchange quads, so that lane (n, h) holds rows 16 g + 8 h .. +7
// (g = 0, 1) and writes two 16-byte pieces: with 8-byte pieces at a row pitch of kilobytes L2 does
// not always merge the partial sectors before they are evicted.
__device__ __forceinline__ void store_block32_bf16(__bf16* dst, const f32x16& acc, float mul, int h, bool ok) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  uint32_t w[4][2];  // [q][half of the quad] as packed bf16 pairs
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      bf16x2_t pr;
      pr[0] = (__bf16)(acc[4 * q + 2 * j] * mul);
      pr[1] = (__bf16)(acc[4 * q + 2 * j + 1] * mul);
      w[q][j] = __builtin_bit_cast(uint32_t, pr);
    }
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    uint32_t lo[2], hi[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      // r[0] = {a[0..31], b[0..31]}, r[1] = {a[32..63], b[32..63]} with a = quad 2g, b = quad 2g+1:
      // lanes h = 0 get rows 16g+0..3 (own) and 16g+4..7 (partner's quad 2g);
      // lanes h = 1 get rows 16g+8..11 (partner's quad 2g+1) and 16g+12..15 (own)
      auto r = __builtin_amdgcn_permlane32_swap(w[2 * g][j], w[2 * g + 1][j], false, false);
      lo[j] = r[0];
      hi[j] = r[1];
    }
    u32x4 out = {lo[0], lo[1], hi[0], hi[1]};
    if (ok) *reinterpret_cast<u32x4*>(dst + 16 * g + 8 * h) = out;  // (every lane takes part in the exchange)
  }
}

// ---- LDS tile layout -------------------------------------------------------------------
// A tile is ROWS x D bf16, row pitch D*2 bytes, no padding.  The 16-byte chunk c of row r
// sits at chunk position c ^ swz(r), which keeps both access patterns spread over the
// banks: 16 lanes reading the same chunk of 16 consecutive rows (MFMA operand rows), and
// the transpose loads that read 4 consecutive rows x 64 contiguous bytes.
template <int D>
__device__ __forceinline__ int swz(int r) {
  int f = ((r & 3) << 2) | (((r >> 2) ^ r) & 3);
  return f & (D / 8 - 1);
}
template <int D>
__device__ __forceinline__ int tile_off(int r, int chunk) {  // byte offset of 16-byte chunk
  return r * (D * 2) + ((chunk ^ swz<D>(r)) << 4);
}

__device__ __forceinline__ bf16x8 lds_read8(const char* base, int off) {
  return *reinterpret_cast<const bf16x8*>(base + off);
}

// Transpose load: returns 4 bf16 = rows r0..r0+3 (see header) of this lane's column.
__device__ __forceinline__ bf16x4 lds_read_tr4(const char* p) {
  typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
  i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(p));
  return __builtin_bit_cast(bf16x4, v);
}
__device__ __forceinline__ bf16x8 cat4(bf16x4 a, bf16x4 b) {
  return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Byte offset this lane passes to the transpose load so that, for a tile in the swizzled
// layout, it receives rows r0 + {0..3} of column (c0 + lane % 16), where c0 is a multiple of 16.
template <int D>
__device__ __forceinline__ int tr_off(int lane, int r0, int c0) {
  int L = lane & 15;
  int row = r0 + (L >> 2);
  int col = c0 + ((L & 3) << 2);
  return row * (D * 2) + (((col >> 3) ^ swz<D>(row)) << 4) + ((col & 4) << 1);
}

// ---- global -> register -> LDS tile copies --------------------------------------------
// A ROWS x D tile is ROWS * D/8 chunks of 16 bytes; thread t owns chunks t, t+256, ...
template <int ROWS, int D>
struct TileRegs {
  static constexpr int N = ROWS * (D / 8) / kThreads;
  u32x4 r[N];
};

// Rows row0 .. row0+ROWS-1 of a [*, heads, D] tensor (head already folded into `base`,
// row stride `stride` elements); rows past row_last are clamped to row_last so that no
// load leaves the tensor (their values are masked by the caller).
template <int ROWS, int D>
__device__ __forceinline__ void tile_load(TileRegs<ROWS, D>& t, const __bf16* base, int64_t stride,
                                          int64_t row0, int64_t row_last, int tid) {
#pragma unroll
  for (int i = 0; i < TileRegs<ROWS, D>::N; ++i) {
    int c = tid + i * kThreads;
    int r = c / (D / 8), ch = c % (D / 8);
    int64_t row = row0 + r;
    row = row < row_last ? row : row_last;
    t.r[i] = *reinterpret_cast<const u32x4*>(base + row * stride + ch * 8);
  }
}
template <int ROWS, int D>
__device__ __forceinline__ void tile_store(const TileRegs<ROWS, D>& t, char* lds, int tid) {
#pragma unroll
  for (int i = 0; i < TileRegs<ROWS, D>::N; ++i) {
    int c = tid + i * kThreads;
    int r = c / (D / 8), ch = c % (D / 8);
    *reinterpret_cast<u32x4*>(lds + tile_off<D>(r, ch)) = t.r[i];
  }
}

// ---- global -> LDS tile copies without a register stop -----------------------------------
// global_load_lds_dwordx4 writes lane L's 16 bytes to LDS at M0 + 16 L, so one wave
// instruction fills 1 KiB = 64 consecutive chunk positions of the tile.  The swizzle is
// applied on the global side: the lane that owns chunk POSITION pc of row r fetches the
// LOGICAL chunk pc ^ swz(r) of that row (still inside the row's contiguous D*2 bytes).
// A 64-row tile takes 64*D*2/1024 wave instructions, dealt round-robin to the 4 waves.
//
// The instruction is issued from inline assembly on purpose: written as a builtin, the
// compiler cannot tell the LDS stage being filled from the stage being read and drains
// every outstanding copy (s_waitcnt vmcnt(0)) in front of the first LDS read that follows,
// which serialises the prefetch with the arithmetic.  The price is that the kernel itself
// must call async_wait_all() before the barrier that publishes a filled stage.  M0 is written
// without telling the compiler (it is a reserved register that cannot be listed as a clobber);
// nothing else in these kernels uses M0.
// Values that are the same in every lane but that the compiler cannot prove uniform (they
// came through LDS or a per-lane load) are moved to scalar registers explicitly; for values it
// already keeps in scalar registers this folds away.
__device__ __forceinline__ uint32_t uniform(uint32_t x) { return (uint32_t)__builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ const char* uniform(const char* p) {
  const uint64_t x = (uint64_t)p;
  // the builtin returns a signed int: narrow to 32 unsigned bits before widening, or the low
  // word's sign bit smears over the high word
  const uint64_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)x);
  const uint64_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
  return (const char*)(lo | (hi << 32));
}

__device__ __forceinline__ int64_t uniform(int64_t x) { return (int64_t)(uintptr_t)uniform((const char*)(uintptr_t)x); }

__device__ __forceinline__ void async_copy16(uint32_t voffset, const char* sbase, uint32_t lds_addr) {
  sbase = uniform(sbase);
  lds_addr = uniform(lds_addr);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(voffset), "s"(sbase), "s"(lds_addr)
               : "memory");
}
// The same for data that is read once (non-temporal: the lines are the first to leave L2 again).
__device__ __forceinline__ void async_copy16_stream(uint32_t voffset, const char* sbase, uint32_t lds_addr) {
  sbase = uniform(sbase);
  lds_addr = uniform(lds_addr);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
               :
               : "v"(voffset), "s"(sbase), "s"(lds_addr)
               : "memory");
}
__device__ __forceinline__ void async_wait_all() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Makes the compiler treat `x` as consumed here, so that the wait for the global load that
// produces it is placed here and not at its first real use.  Needed before a pipelined loop:
// a wait left inside the loop body would, from the second trip on, drain the asynchronous
// copies issued at the top of the trip instead (the hardware counter is shared).
template <typename T>
__device__ __forceinline__ void consume(const T& x) {
  asm volatile("" ::"v"(x));
}

__device__ __forceinline__ uint32_t lds_address(const void* p) {  // LDS byte address of a pointer into shared memory
  return (uint32_t)(uintptr_t)p;
}

template <int D, int WAVES = 4>
struct AsyncTile {
  static constexpr int CPR = D / 8;          // 16-byte chunks per row
  static constexpr int RPI = 64 / CPR;       // rows per wave instruction
  static constexpr int NI = 64 / RPI / WAVES;  // instructions per wave per tile
  int row0;             // row this lane fetches in instruction 0 (instruction i adds WAVES * RPI * i)
  uint32_t chunk_byte;  // byte offset of its logical chunk inside the row
  uint32_t voff;        // row0 * pitch + chunk_byte
  uint32_t pitch;       // bytes between consecutive rows (< 2^24)
  int wave;             // wave index, uniform

  __device__ __forceinline__ void init(int tid, int64_t pitch_bytes) {
    const int lane = tid & 63;
    wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    row0 = wave * RPI + lane / CPR;
    static_assert((WAVES * RPI) % 16 == 0, "the swizzle of a lane's row must not change from one instruction to the next");
    chunk_byte = ((lane % CPR) ^ swz<D>(row0)) << 4;  // swz depends on row & 15 only; WAVES*RPI*i is a multiple of 16
    pitch = (uint32_t)pitch_bytes;
    voff = (uint32_t)row0 * pitch + chunk_byte;
  }

  // Copies 64 full rows starting at `g` (wave-uniform) into the LDS tile at byte address `lds`.
  __device__ __forceinline__ void load_full(uint32_t lds, const char* g) const {
#pragma unroll
    for (int i = 0; i < NI; ++i) load_full_piece(lds, g, i);
  }
  // One of the NI instructions of load_full, for callers that spread them over their arithmetic
  // (a wave issues in order, and the memory pipeline accepts about 1 KiB per 16 cycles per CU).
  __device__ __forceinline__ void load_full_piece(uint32_t lds, const char* g, int i) const {
    async_copy16(voff, g + (uint64_t)(WAVES * RPI * i) * pitch, lds + (i * WAVES + wave) * 1024);
  }
  // Same when only rows [0, rows_valid) exist: later rows repeat row rows_valid-1 so that no
  // load leaves the tensor (their values are masked by the caller).  1 <= rows_valid <= 64.
  __device__ __forceinline__ void load_partial(uint32_t lds, const char* g, int rows_valid) const {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      int r = row0 + WAVES * RPI * i;
      r = r < rows_valid ? r : rows_valid - 1;
      async_copy16((uint32_t)r * pitch + chunk_byte, g, lds + (i * WAVES + wave) * 1024);
    }
  }
  __device__ __forceinline__ void load(uint32_t lds, const char* g, int rows_valid) const {
    if (rows_valid >= 64) load_full(lds, g);
    else load_partial(lds, g, rows_valid);
  }
};

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// x * f, element by element, rounded back to bf16 (nearest even).
__device__ __forceinline__ bf16x8 scale_frag(bf16x8 x, float f) {
  bf16x8 r;
#pragma unroll
  for (int t = 0; t < 8; ++t) r[t] = (__bf16)((float)x[t] * f);
  return r;
}

// Rounds two floats to bf16 (nearest even) into one register.
__device__ __forceinline__ bf16x2 pack_bf16(float a, float b) {
  bf16x2 r;
  r[0] = (__bf16)a;
  r[1] = (__bf16)b;
  return r;
}
// acc + p[0] + p[1] in fp32 (v_dot2c_f32_bf16 against a pair of ones).
__device__ __forceinline__ float add_pair(bf16x2 p, float acc) {
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  return __builtin_amdgcn_fdot2_f32_bf16(p, ones, acc, false);
}
// Four bf16 pairs -> one 8-element MFMA operand.
__device__ __forceinline__ bf16x8 cat_pairs(bf16x2 a, bf16x2 b, bf16x2 c, bf16x2 d) {
  u32x4 w = {__builtin_bit_cast(uint32_t, a), __builtin_bit_cast(uint32_t, b), __builtin_bit_cast(uint32_t, c),
             __builtin_bit_cast(uint32_t, d)};
  return __builtin_bit_cast(bf16x8, w);
}

// ---- workgroup -> (batch, head, document, tile) ----------------------------------------
struct TileCoord {
  int b, h;
  int64_t doc_begin, doc_end;  // token range of the document
  int64_t t0;                  // first token of the tile
  bool valid;
};

// Tiles of `TS` tokens never straddle documents.  `w` is the item number a persistent workgroup
// drew from its queue (tile_queue.hpp): item w belongs to the list of XCD w & 7 and is that
// list's entry number w >> 3.  When B*H is a multiple of 8, list x holds the heads x, x+8, ... .
// Its first part walks the heads one after the other, the heavier 5/8 of each head's tiles from
// the heaviest down: the workgroups of an XCD then stream the SAME head's K/V (or Q/dO) through
// its L2 nearly in lock-step, and each is fetched from HBM once per group of co-resident tiles.
// Its last part holds the lighter 3/8 of the tiles of all its heads, interleaved by weight, so that
// the items still running when the lists run empty are small (the kernel ends when the slowest
// workgroup does).  Otherwise (B*H not a multiple of 8) there is one list and heads simply
// alternate (head = w % (B*H)).  `heavy_last` says whether high tile numbers carry the most work
// (forward and dq: causal rows late in a document see more keys).
// `scratch`: 2 * THREADS / 64 + 2 ints of LDS (THREADS = workgroup size).
template <int TS, int THREADS = kThreads>
__device__ __forceinline__ TileCoord decode_tile(const AttnParams& p, int heads, bool heavy_last, int* scratch, int w, int tid) {
  constexpr int NW = THREADS / 64;
  TileCoord c;
  // (the divisors below are the same for every item of a launch; they are made opaque so that a persistent kernel
  // does not compute their reciprocals ahead of its item loop and keep them in registers through it)
  auto opaque = [](int x) { asm volatile("" : "+s"(x)); return x; };
  heads = opaque(heads);
  const int nH = opaque((int)p.B * heads);
  int hh, t;
  if (nH % 8 == 0) {
    const int xcd = w & 7, slot = w >> 3;
    const int hpx = opaque(nH / 8);                        // heads per list
    const int heavy = opaque(p.q_heavy);                   // tiles per head in the head-by-head part
    if (slot < heavy * hpx) { hh = xcd + 8 * (slot / heavy); t = slot % heavy; }
    else { const int r = slot - heavy * hpx; hh = xcd + 8 * (r % hpx); t = heavy + r / hpx; }
  } else {
    hh = w % nH;
    t = w / nH;
  }
  if (heavy_last) t = p.tiles - 1 - t;
  c.b = hh / heads;
  c.h = hh % heads;
  if (p.cu == nullptr) {
    c.doc_begin = 0;
    c.doc_end = p.S;
    c.t0 = (int64_t)t * TS;
    c.valid = c.t0 < p.S;
    return c;
  }
  // Packed: find the document whose tile range contains t.  Thread i counts the tiles of
  // documents i, i+256, ... in rounds of 256 documents with a block-wide scan per round.
  // (`tid` is the caller's copy of the thread index: persistent kernels pass an opaque one, so that nothing
  // below is computed ahead of their item loop and kept in registers through it)
  int lane = tid & 63, wv = tid >> 6;
  int* s_wave = scratch;       // [NW] wave totals
  int* s_res = scratch + NW;   // [0] doc index or -1, [1] tiles before that doc
  if (tid == 0) { s_res[0] = -1; s_res[1] = 0; }
  __syncthreads();
  int before = 0;  // tiles of all documents in earlier rounds
  for (int base = 0; base < p.num_docs; base += THREADS) {
    int d = base + tid;
    int nt = 0;
    if (d < p.num_docs) nt = (p.cu[d + 1] - p.cu[d] + TS - 1) / TS;
    int inc = nt;  // inclusive scan inside the wave
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
      int y = __shfl_up(inc, s, 64);
      if (lane >= s) inc += y;
    }
    if (lane == 63) s_wave[wv] = inc;
    __syncthreads();
    int woff = 0, total = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) { int x = s_wave[i]; if (i < wv) woff += x; total += x; }
    int excl = before + woff + inc - nt;
    if (nt > 0 && t >= excl && t < excl + nt) { s_res[0] = d; s_res[1] = excl; }
    __syncthreads();
    before += total;
    if (s_res[0] >= 0 || t < before) break;
  }
  __syncthreads();
  int d = s_res[0];
  if (d < 0) { c.valid = false; c.doc_begin = c.doc_end = c.t0 = 0; return c; }
  c.doc_begin = p.cu[d];
  c.doc_end = p.cu[d + 1];
  c.t0 = c.doc_begin + (int64_t)(t - s_res[1]) * TS;
  c.valid = true;
  return c;
}

}  // namespace ie
