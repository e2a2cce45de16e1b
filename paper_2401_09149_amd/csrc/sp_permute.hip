// The eight local re-layouts either side of the sequence-parallel all-to-alls (include/ie_sp.h;
// Sec. 2.4 "SP-2", Sec. 3.2.2 "Sequence Parallelism").  Every one of them moves contiguous runs of
// Hl*D bf16 values (one token's heads of one head group) between two 4-level strided layouts
// indexed by (peer p, batch b, token s of the slice, position in the run), so one kernel serves
// all: a "plane" descriptor gives the strides of both sides, and the q, k and v planes of the
// fused tensors are three planes of one launch.  The work is a pure copy: HBM bandwidth bounds
// it (2 bytes moved per byte of tensor), so the kernel moves 16 bytes per lane per access with
// streaming (nontemporal) loads and stores, and does its only division once per lane.
#include "../../include/ie_sp.h"

#include <hip/hip_runtime.h>

#include "launch.hpp"

namespace {

typedef uint32_t unit_t __attribute__((ext_vector_type(4)));   // 16 bytes = 8 bf16

// Offsets in units: run (p, b, s) of the plane starts at src + p*sp + b*sb + s*ss and goes to
// dst + p*dp + b*db + s*ds; a run is `wu` units long.
struct Plane {
  const unit_t* src;
  unit_t* dst;
  int64_t sp, sb, ss;
  int64_t dp, db, ds;
  uint32_t wu;     // units per run
  uint32_t rows;   // runs (tokens) per workgroup
};

struct PermuteParams {
  Plane pl[3];
  int64_t Sl;
  uint32_t B;
};

constexpr int kThreads = 256;
// Measured on cold buffers (1.2 GB ring): 16 KiB per workgroup with two loads in flight per lane moves
// 5.7-5.9 TB/s; 64 KiB tiles lose 5 %, plain (cached) loads or stores 3-5 %.
constexpr int kUnroll = 2;
constexpr uint32_t kTileUnits = 1024;   // 16 KiB per workgroup

// grid: x = tiles of `rows` tokens, y = p*B + b, z = plane
__global__ __launch_bounds__(kThreads) void sp_permute_kernel(PermuteParams prm) {
  const Plane& pl = prm.pl[blockIdx.z];
  const int64_t s0 = (int64_t)blockIdx.x * pl.rows;
  if (s0 >= prm.Sl) return;   // planes with wider runs have fewer tiles
  const int64_t left = prm.Sl - s0;
  const uint32_t rows = left < (int64_t)pl.rows ? (uint32_t)left : pl.rows;
  const uint32_t p = blockIdx.y / prm.B, b = blockIdx.y % prm.B;
  const unit_t* src = pl.src + p * pl.sp + b * pl.sb + s0 * pl.ss;
  unit_t* dst = pl.dst + p * pl.dp + b * pl.db + s0 * pl.ds;
  const uint32_t wu = pl.wu;
  const uint32_t n = rows * wu;
  // lane's unit u = tid + 256*i lies in run `row` at position `col`; advancing u by 256 advances
  // (row, col) by (dr, dc) with a carry
  uint32_t row = threadIdx.x / wu, col = threadIdx.x % wu;
  const uint32_t dr = kThreads / wu, dc = kThreads % wu;
  for (uint32_t u = threadIdx.x; u < n; u += kThreads * kUnroll) {
    unit_t val[kUnroll];
    int64_t doff[kUnroll];
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      const bool ok = u + i * kThreads < n;
      doff[i] = ok ? (int64_t)row * pl.ds + col : -1;
      if (ok) val[i] = __builtin_nontemporal_load(src + ((int64_t)row * pl.ss + col));
      row += dr;
      col += dc;
      if (col >= wu) { col -= wu; ++row; }
    }
#pragma unroll
    for (int i = 0; i < kUnroll; ++i)
      if (doff[i] >= 0) __builtin_nontemporal_store(val[i], dst + doff[i]);
  }
}

constexpr int64_t kMaxElems = (int64_t)1 << 40;

struct Shape {
  int64_t B, Sl;
  int64_t wq, wk;   // units per run of the q plane / of the k and v planes (per-peer heads)
  int64_t P;
};

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

int check(int64_t B, int64_t Sl, int32_t Hq, int32_t Hkv, int32_t D, int32_t P, Shape* s) {
  if (B <= 0 || Sl <= 0 || Hq <= 0 || Hkv <= 0 || P <= 0) return IE_ERR_SHAPE;
  if (Hq % P != 0 || Hkv % P != 0) return IE_ERR_SHAPE;
  if (D <= 0 || D % 8 != 0) return IE_ERR_UNSUPPORTED;
  // the largest buffer is the fused one, B*Sl*(Hq+2Hkv)*D elements, or a q-sized one of B*P*Sl*(Hq/P)*D
  const int64_t heads = (int64_t)Hq + 2 * (int64_t)Hkv;
  if (B > kMaxElems / Sl || B * Sl > kMaxElems / heads || B * Sl * heads > kMaxElems / D) return IE_ERR_SHAPE;
  if ((int64_t)P * B > 65535) return IE_ERR_SHAPE;   // grid y
  s->B = B; s->Sl = Sl; s->P = P;
  s->wq = (int64_t)(Hq / P) * D / 8;
  s->wk = (int64_t)(Hkv / P) * D / 8;
  return IE_OK;
}

void set_plane(Plane& pl, const void* src, int64_t src_base, int64_t sp, int64_t sb, int64_t ss, void* dst,
               int64_t dst_base, int64_t dp, int64_t db, int64_t ds, int64_t wu) {
  pl.src = static_cast<const unit_t*>(src) + src_base;
  pl.dst = static_cast<unit_t*>(dst) + dst_base;
  pl.sp = sp; pl.sb = sb; pl.ss = ss;
  pl.dp = dp; pl.db = db; pl.ds = ds;
  pl.wu = (uint32_t)wu;
  pl.rows = wu >= kTileUnits ? 1u : kTileUnits / (uint32_t)wu;
}

void swap_sides(Plane& pl) {
  Plane o = pl;
  pl.src = o.dst; pl.dst = const_cast<unit_t*>(o.src);
  pl.sp = o.dp; pl.sb = o.db; pl.ss = o.ds;
  pl.dp = o.sp; pl.db = o.sb; pl.ds = o.ss;
}

int launch(PermuteParams& prm, int nplanes, const Shape& s, bool reverse, void* stream) {
  uint32_t min_rows = prm.pl[0].rows;
  for (int t = 0; t < nplanes; ++t) {
    if (reverse) swap_sides(prm.pl[t]);
    if (prm.pl[t].rows < min_rows) min_rows = prm.pl[t].rows;
  }
  prm.Sl = s.Sl;
  prm.B = (uint32_t)s.B;
  const int64_t tiles = ie::ceil_div(s.Sl, min_rows);
  if (tiles >= ((int64_t)1 << 31)) return IE_ERR_SHAPE;
  dim3 grid((uint32_t)tiles, (uint32_t)(s.P * s.B), (uint32_t)nplanes);
  sp_permute_kernel<<<grid, kThreads, 0, static_cast<hipStream_t>(stream)>>>(prm);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? IE_OK : ie::hip_fail(e);
}

// fused local tensor [B][q | k | v] with all heads  <->  exchange buffer [P][B][q | k | v] with per-peer heads
int qkv_local_and_x(const void* local, void* x, const Shape& s, bool reverse, void* stream) {
  const int64_t Wq = s.wq * s.P, Wk = s.wk * s.P;                 // units per token, all heads
  const int64_t Lb = s.Sl * (Wq + 2 * Wk), Xb = s.Sl * (s.wq + 2 * s.wk);
  const int64_t w[3] = {s.wq, s.wk, s.wk}, W[3] = {Wq, Wk, Wk};
  const int64_t lbase[3] = {0, s.Sl * Wq, s.Sl * (Wq + Wk)};
  const int64_t xbase[3] = {0, s.Sl * s.wq, s.Sl * (s.wq + s.wk)};
  PermuteParams prm;
  for (int t = 0; t < 3; ++t)
    set_plane(prm.pl[t], local, lbase[t], w[t], Lb, W[t], x, xbase[t], s.B * Xb, Xb, w[t], w[t]);
  return launch(prm, 3, s, reverse, stream);
}

// exchange buffer [P][B][q | k | v]  <->  three attention operands [B][P*Sl][Hl][D]
int x_and_qkv(const void* x, void* const t3[3], const Shape& s, bool reverse, void* stream) {
  const int64_t Xb = s.Sl * (s.wq + 2 * s.wk);
  const int64_t w[3] = {s.wq, s.wk, s.wk};
  const int64_t xbase[3] = {0, s.Sl * s.wq, s.Sl * (s.wq + s.wk)};
  PermuteParams prm;
  for (int t = 0; t < 3; ++t)
    set_plane(prm.pl[t], x, xbase[t], s.B * Xb, Xb, w[t], t3[t], 0, s.Sl * w[t], s.P * s.Sl * w[t], w[t], w[t]);
  return launch(prm, 3, s, reverse, stream);
}

// attention operand [B][P*Sl][Hql][D]  <->  exchange buffer [P][B][Sl][Hql][D]
int o_and_x(const void* o, void* x, const Shape& s, bool reverse, void* stream) {
  PermuteParams prm;
  set_plane(prm.pl[0], o, 0, s.Sl * s.wq, s.P * s.Sl * s.wq, s.wq, x, 0, s.B * s.Sl * s.wq, s.Sl * s.wq, s.wq, s.wq);
  return launch(prm, 1, s, reverse, stream);
}

// exchange buffer [P][B][Sl][Hql][D]  <->  local tensor [B][Sl][Hq][D]
int x_and_o_local(const void* x, void* local, const Shape& s, bool reverse, void* stream) {
  PermuteParams prm;
  const int64_t Wq = s.wq * s.P;
  set_plane(prm.pl[0], x, 0, s.B * s.Sl * s.wq, s.Sl * s.wq, s.wq, local, 0, s.wq, s.Sl * Wq, Wq, s.wq);
  return launch(prm, 1, s, reverse, stream);
}

}  // namespace

extern "C" {

int ie_sp_pack_qkv(const void* qkv_local, void* xqkv, int64_t B, int64_t Sl, int32_t Hq, int32_t Hkv, int32_t D,
                   int32_t P, void* stream) {
  if (!qkv_local || !xqkv) return IE_ERR_NULL;
  Shape s;
  if (int rc = check(B, Sl, Hq, Hkv, D, P, &s)) return rc;
  if (!aligned16(qkv_local) || !aligned16(xqkv)) return IE_ERR_ALIGN;
  return qkv_local_and_x(qkv_local, xqkv, s, false, stream);
}

int ie_sp_unpack_dqkv(const void* xqkv, void* dqkv_local, int64_t B, int64_t Sl, int32_t Hq, int32_t Hkv, int32_t D,
                      int32_t P, void* stream) {
  if (!xqkv || !dqkv_local) return IE_ERR_NULL;
  Shape s;
  if (int rc = check(B, Sl, Hq, Hkv, D, P, &s)) return rc;
  if (!aligned16(xqkv) || !aligned16(dqkv_local)) return IE_ERR_ALIGN;
  return qkv_local_and_x(dqkv_local, const_cast<void*>(xqkv), s, true, stream);
}

int ie_sp_unpack_qkv(const void* xqkv, void* q, void* k, void* v, int64_t B, int64_t Sl, int32_t Hq, int32_t Hkv,
                     int32_t D, int32_t P, void* stream) {
  if (!xqkv || !q || !k || !v) return IE_ERR_NULL;
  Shape s;
  if (int rc = check(B, Sl, Hq, Hkv, D, P, &s)) return rc;
  if (!aligned16(xqkv) || !aligned16(q) || !aligned16(k) || !aligned16(v)) return IE_ERR_ALIGN;
  void* const t3[3] = {q, k, v};
  return x_and_qkv(xqkv, t3, s, false, stream);
}

int ie_sp_pack_dqkv(const void* dq, const void* dk, const void* dv, void* xqkv, int64_t B, int64_t Sl, int32_t Hq,
                    int32_t Hkv, int32_t D, int32_t P, void* stream) {
  if (!dq || !dk || !dv || !xqkv) return IE_ERR_NULL;
  Shape s;
  if (int rc = check(B, Sl, Hq, Hkv, D, P, &s)) return rc;
  if (!aligned16(xqkv) || !aligned16(dq) || !aligned16(dk) || !aligned16(dv)) return IE_ERR_ALIGN;
  void* const t3[3] = {const_cast<void*>(dq), const_cast<void*>(dk), const_cast<void*>(dv)};
  return x_and_qkv(xqkv, t3, s, true, stream);
}

int ie_sp_pack_o(const void* o, void* xo, int64_t B, int64_t Sl, int32_t Hq, int32_t D, int32_t P, void* stream) {
  if (!o || !xo) return IE_ERR_NULL;
  Shape s;
  if (int rc = check(B, Sl, Hq, Hq, D, P, &s)) return rc;
  if (!aligned16(o) || !aligned16(xo)) return IE_ERR_ALIGN;
  return o_and_x(o, xo, s, false, stream);
}

int ie_sp_unpack_do(const void* xo, void* dout, int64_t B, int64_t Sl, int32_t Hq, int32_t D, int32_t P,
                    void* stream) {
  if (!xo || !dout) return IE_ERR_NULL;
  Shape s;
  if (int rc = check(B, Sl, Hq, Hq, D, P, &s)) return rc;
  if (!aligned16(xo) || !aligned16(dout)) return IE_ERR_ALIGN;
  return o_and_x(dout, const_cast<void*>(xo), s, true, stream);
}

int ie_sp_unpack_o(const void* xo, void* o_local, int64_t B, int64_t Sl, int32_t Hq, int32_t D, int32_t P,
                   void* stream) {
  if (!xo || !o_local) return IE_ERR_NULL;
  Shape s;
  if (int rc = check(B, Sl, Hq, Hq, D, P, &s)) return rc;
  if (!aligned16(xo) || !aligned16(o_local)) return IE_ERR_ALIGN;
  return x_and_o_local(xo, o_local, s, false, stream);
}

int ie_sp_pack_do(const void* dout_local, void* xo, int64_t B, int64_t Sl, int32_t Hq, int32_t D, int32_t P,
                  void* stream) {
  if (!dout_local || !xo) return IE_ERR_NULL;
  Shape s;
  if (int rc = check(B, Sl, Hq, Hq, D, P, &s)) return rc;
  if (!aligned16(dout_local) || !aligned16(xo)) return IE_ERR_ALIGN;
  return x_and_o_local(const_cast<void*>(xo), const_cast<void*>(dout_local), s, true, stream);
}

}  // extern "C"
