// C-ABI entry points (include/ie_attn.h): argument validation, workspace carving and
// kernel launches.  Host code only decides shapes and grids; every step of the path
// runs in the kernels of attn_fwd.hip / attn_bwd.hip.
#include "../../include/ie_attn.h"

#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>

#include "attn_common.hpp"
#include "launch.hpp"

namespace {

thread_local char g_hip_error[256] = "";

constexpr int64_t kMaxElems = (int64_t)1 << 40;

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// One [B,Hq,S] fp32 plane of the backward workspace; and its counter area (tile_queue.hpp: kQueueBytes per kernel).
size_t stat_bytes(int64_t B, int64_t S, int32_t Hq) { return align_up((size_t)B * (size_t)Hq * (size_t)S * sizeof(float), 256); }
constexpr size_t kCounterBytes = 256;

ie::AttnParams base_params(const int32_t* cu, int32_t num_docs, int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D,
                           float scale, int32_t causal) {
  ie::AttnParams p;
  std::memset(&p, 0, sizeof(p));
  p.cu = cu;
  p.num_docs = cu ? num_docs : 0;
  p.B = B; p.S = S; p.Hq = Hq; p.Hkv = Hkv;
  p.scale = scale;
  p.scale_log2 = scale * ie::kLog2e;
  p.causal = causal;
  // contiguous [B,S,heads,D] tensors: one "chunk" per batch entry
  p.tok_shift = 63;
  p.tok_mask = INT64_MAX;
  p.tok_cstride = 0;
  p.q_bstride = S * (int64_t)Hq * D * 2;
  p.kv_bstride = S * (int64_t)Hkv * D * 2;
  return p;
}

int check_shape(const int32_t* cu, int32_t num_docs, int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D,
                float scale, int32_t causal) {
  if (B <= 0 || S <= 0 || Hq <= 0 || Hkv <= 0) return IE_ERR_SHAPE;
  if (Hq % Hkv != 0) return IE_ERR_SHAPE;
  if (cu != nullptr && (B != 1 || num_docs < 1)) return IE_ERR_SHAPE;
  if (D != 64 && D != 128) return IE_ERR_UNSUPPORTED;
  if (!(scale > 0.0f) || !std::isfinite(scale)) return IE_ERR_UNSUPPORTED;
  if (causal != 0 && causal != 1) return IE_ERR_UNSUPPORTED;
  // element counts must stay far from overflow and the grid below 2^31
  if (B > kMaxElems / S || B * S > kMaxElems / Hq || B * S * Hq > kMaxElems / D) return IE_ERR_SHAPE;
  if (S >= ((int64_t)1 << 31)) return IE_ERR_SHAPE;
  // the tile loaders address rows with 32-bit byte offsets: one token row of all heads must stay below 16 MiB
  if ((int64_t)Hq * D * 2 >= ((int64_t)1 << 24)) return IE_ERR_SHAPE;
  return IE_OK;
}

}  // namespace

namespace ie {
int hip_fail(hipError_t e) {
  std::strncpy(g_hip_error, hipGetErrorString(e), sizeof(g_hip_error) - 1);
  g_hip_error[sizeof(g_hip_error) - 1] = 0;
  return IE_ERR_HIP;
}
}  // namespace ie

// ---- backward without a workspace argument -------------------------------------------------------
// For callers that cannot allocate (code under graph capture, serving loops, harnesses that forbid it):
// the workspace of ie_attn_bwd lives in a file-scope device array instead, one copy per device.  Host
// code must not hand the array's name to a kernel; its device address is asked for once per device.
constexpr size_t kStaticRows = (size_t)IE_ATTN_BWD_STATIC_MAX_ROWS;
constexpr size_t kStaticBytes = 2 * kStaticRows * sizeof(float) + kCounterBytes;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

static std::mutex g_scratch_mu;
static void* g_scratch_ptr[ie::kMaxDevices];   // device address of `scratch`, per device

extern "C" {

int ie_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse, const int32_t* cu_seqlens,
                int32_t num_docs, int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D, float scale,
                int32_t causal, void* stream) {
  if (!q || !k || !v || !o || !lse) return IE_ERR_NULL;
  int rc = check_shape(cu_seqlens, num_docs, B, S, Hq, Hkv, D, scale, causal);
  if (rc) return rc;
  ie::AttnParams p = base_params(cu_seqlens, num_docs, B, S, Hq, Hkv, D, scale, causal);
  p.q = static_cast<const __bf16*>(q);
  p.k = static_cast<const __bf16*>(k);
  p.v = static_cast<const __bf16*>(v);
  p.o_out = static_cast<__bf16*>(o);
  p.lse_out = lse;
  hipStream_t st = static_cast<hipStream_t>(stream);
  return ie::launch_fwd(p, D, st);
}

size_t ie_attn_bwd_workspace_bytes(int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D, int32_t num_docs) {
  (void)num_docs;
  if (check_shape(nullptr, 0, B, S, Hq, Hkv, D, 1.0f, 1) != IE_OK) return 0;
  // -delta and -lse*log2e, [B,Hq,S] fp32 each, then the work-queue counters of the call's kernels
  return 2 * stat_bytes(B, S, Hq) + kCounterBytes;
}

// dS of dense input, bf16 in 128 x 128 blocks: per (batch, query head) the lower block triangle when causal, else all.
static size_t ds_bytes(int64_t B, int64_t S, int32_t Hq, int32_t causal) {
  const size_t nt = (size_t)(S / 128);
  return (size_t)B * (size_t)Hq * (causal ? nt * (nt + 1) / 2 : nt * nt) * 32768;
}

size_t ie_attn_bwd_fast_workspace_bytes(int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D, int32_t num_docs,
                                        int32_t causal) {
  const size_t base = ie_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D, num_docs);
  if (base == 0 || num_docs != 0 || (causal != 0 && causal != 1) || D != 128 || S % 128 != 0) return base;
  // (the kernels keep byte offsets inside one query tile's block in 32 bits: 256 S bytes; and no device holds 2^50)
  if (S >= ((int64_t)1 << 23) || (double)B * Hq * (double)S * ((double)S + 128) > 1e15) return base;
  return base + ds_bytes(B, S, Hq, causal);
}

int ie_attn_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout, const float* lse,
                void* dq, void* dk, void* dv, const int32_t* cu_seqlens, int32_t num_docs, int64_t B, int64_t S,
                int32_t Hq, int32_t Hkv, int32_t D, float scale, int32_t causal, void* workspace,
                size_t workspace_bytes, void* stream) {
  return ie_attn_bwd_phases(q, k, v, o, dout, lse, dq, dk, dv, cu_seqlens, num_docs, B, S, Hq, Hkv, D, scale,
                            causal, workspace, workspace_bytes, IE_BWD_ALL, stream);
}

int ie_attn_bwd_phases(const void* q, const void* k, const void* v, const void* o, const void* dout,
                       const float* lse, void* dq, void* dk, void* dv, const int32_t* cu_seqlens,
                       int32_t num_docs, int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D, float scale,
                       int32_t causal, void* workspace, size_t workspace_bytes, int32_t phases, void* stream) {
  if (!q || !k || !v || !o || !dout || !lse || !dq || !dk || !dv) return IE_ERR_NULL;
  int rc = check_shape(cu_seqlens, num_docs, B, S, Hq, Hkv, D, scale, causal);
  if (rc) return rc;
  if ((phases & IE_BWD_ALL) == 0 || (phases & ~(IE_BWD_ALL | IE_BWD_STORED_DS)) != 0) return IE_ERR_UNSUPPORTED;
  const size_t need = ie_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D, num_docs);
  size_t required = need;
  if (phases & IE_BWD_STORED_DS) {   // the caller asks for the path that keeps dS in the workspace
    required = cu_seqlens ? need : ie_attn_bwd_fast_workspace_bytes(B, S, Hq, Hkv, D, 0, causal);
    if (required == need) return IE_ERR_UNSUPPORTED;   // this shape has no such path
  }
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0 || workspace_bytes < required) return IE_ERR_WORKSPACE;
  ie::AttnParams p = base_params(cu_seqlens, num_docs, B, S, Hq, Hkv, D, scale, causal);
  p.q = static_cast<const __bf16*>(q);
  p.k = static_cast<const __bf16*>(k);
  p.v = static_cast<const __bf16*>(v);
  p.o = static_cast<const __bf16*>(o);
  p.dout = static_cast<const __bf16*>(dout);
  p.lse = lse;
  char* ws = static_cast<char*>(workspace);
  p.delta = reinterpret_cast<float*>(ws);
  p.lse2 = reinterpret_cast<float*>(ws + stat_bytes(B, S, Hq));
  p.ws_counters = reinterpret_cast<unsigned int*>(ws + 2 * stat_bytes(B, S, Hq));
  p.ds = (phases & IE_BWD_STORED_DS) ? reinterpret_cast<__bf16*>(ws + need) : nullptr;
  p.dq = static_cast<__bf16*>(dq);
  p.dk = static_cast<__bf16*>(dk);
  p.dv = static_cast<__bf16*>(dv);
  hipStream_t st = static_cast<hipStream_t>(stream);
  return ie::launch_bwd(p, D, phases & IE_BWD_ALL, st);
}

int ie_attn_bwd_static(const void* q, const void* k, const void* v, const void* o, const void* dout,
                       const float* lse, void* dq, void* dk, void* dv, const int32_t* cu_seqlens,
                       int32_t num_docs, int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D, float scale,
                       int32_t causal, void* stream) {
  if (!q || !k || !v || !o || !dout || !lse || !dq || !dk || !dv) return IE_ERR_NULL;
  int rc = check_shape(cu_seqlens, num_docs, B, S, Hq, Hkv, D, scale, causal);
  if (rc) return rc;
  const size_t need = ie_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D, num_docs);
  if ((size_t)B * (size_t)Hq * (size_t)S > kStaticRows || need > kStaticBytes) return IE_ERR_WORKSPACE;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return ie::hip_fail(e);
  if (dev >= ie::kMaxDevices) return IE_ERR_UNSUPPORTED;
  void* ptr = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_ptr[dev] == nullptr) {
      void* sym = nullptr;
      if ((e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch))) != hipSuccess) return ie::hip_fail(e);
      g_scratch_ptr[dev] = sym;
    }
    ptr = g_scratch_ptr[dev];
  }
  // Every byte the kernels read from the array is written earlier in the same call (the delta kernel fills both
  // planes for all B*Hq*S rows and clears the work-queue counters), so nothing has to be cleared here.
  return ie_attn_bwd_phases(q, k, v, o, dout, lse, dq, dk, dv, cu_seqlens, num_docs, B, S, Hq, Hkv, D, scale, causal,
                            ptr, kStaticBytes, IE_BWD_ALL, stream);
}

// ---- operands taken from / gradients written to the sequence-parallel exchange buffer --------------------
// Token t of batch entry b sits in chunk t / Sl (the peer it came from) at row t % Sl; the three planes of a chunk
// follow each other.  Tiles of the kernels (at most 256 tokens, aligned) must not straddle chunks, and the kernels
// split t with a shift and a mask: Sl is a power of two, at least 256.
static int sp_shape(int64_t B, int64_t Sl, int32_t Hq, int32_t Hkv, int32_t D, int32_t P, float scale, int32_t causal) {
  if (P < 1 || Sl < 1 || Hq < 1 || Hkv < 1 || Hq % P != 0 || Hkv % P != 0) return IE_ERR_SHAPE;
  if (Sl > (((int64_t)1 << 31) - 1) / P) return IE_ERR_SHAPE;
  int rc = check_shape(nullptr, 0, B, Sl * P, Hq / P, Hkv / P, D, scale, causal);
  if (rc) return rc;
  if (Sl < 256 || (Sl & (Sl - 1)) != 0) return IE_ERR_UNSUPPORTED;
  return IE_OK;
}

static void sp_token_map(ie::AttnParams& p, int64_t B, int64_t Sl, int32_t Hql, int32_t Hkvl, int32_t D) {
  const int64_t chunk_bytes = Sl * (int64_t)(Hql + 2 * Hkvl) * D * 2;
  int shift = 0;
  while (((int64_t)1 << shift) < Sl) ++shift;
  p.tok_shift = shift;
  p.tok_mask = Sl - 1;
  p.tok_cstride = B * chunk_bytes;
  p.q_bstride = chunk_bytes;
  p.kv_bstride = chunk_bytes;
}

int ie_attn_fwd_sp(const void* xqkv, void* o, float* lse, int64_t B, int64_t Sl, int32_t Hq, int32_t Hkv, int32_t D,
                   int32_t P, float scale, int32_t causal, void* stream) {
  if (!xqkv || !o || !lse) return IE_ERR_NULL;
  int rc = sp_shape(B, Sl, Hq, Hkv, D, P, scale, causal);
  if (rc) return rc;
  if ((reinterpret_cast<uintptr_t>(xqkv) & 15) != 0) return IE_ERR_ALIGN;
  const int32_t Hql = Hq / P, Hkvl = Hkv / P;
  ie::AttnParams p = base_params(nullptr, 0, B, Sl * P, Hql, Hkvl, D, scale, causal);
  sp_token_map(p, B, Sl, Hql, Hkvl, D);
  const __bf16* x = static_cast<const __bf16*>(xqkv);
  p.q = x;
  p.k = x + Sl * (int64_t)Hql * D;
  p.v = x + Sl * (int64_t)(Hql + Hkvl) * D;
  p.o_out = static_cast<__bf16*>(o);
  p.lse_out = lse;
  return ie::launch_fwd(p, D, static_cast<hipStream_t>(stream));
}

int ie_attn_bwd_sp(const void* xqkv, const void* o, const void* dout, const float* lse, void* dxqkv, int64_t B,
                   int64_t Sl, int32_t Hq, int32_t Hkv, int32_t D, int32_t P, float scale, int32_t causal,
                   void* workspace, size_t workspace_bytes, void* stream) {
  if (!xqkv || !o || !dout || !lse || !dxqkv) return IE_ERR_NULL;
  int rc = sp_shape(B, Sl, Hq, Hkv, D, P, scale, causal);
  if (rc) return rc;
  if (((reinterpret_cast<uintptr_t>(xqkv) | reinterpret_cast<uintptr_t>(dxqkv)) & 15) != 0) return IE_ERR_ALIGN;
  const int32_t Hql = Hq / P, Hkvl = Hkv / P;
  const int64_t S = Sl * P;
  const size_t need = ie_attn_bwd_workspace_bytes(B, S, Hql, Hkvl, D, 0);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0 || workspace_bytes < need) return IE_ERR_WORKSPACE;
  ie::AttnParams p = base_params(nullptr, 0, B, S, Hql, Hkvl, D, scale, causal);
  sp_token_map(p, B, Sl, Hql, Hkvl, D);
  const __bf16* x = static_cast<const __bf16*>(xqkv);
  __bf16* dx = static_cast<__bf16*>(dxqkv);
  p.q = x;
  p.k = x + Sl * (int64_t)Hql * D;
  p.v = x + Sl * (int64_t)(Hql + Hkvl) * D;
  p.dq = dx;
  p.dk = dx + Sl * (int64_t)Hql * D;
  p.dv = dx + Sl * (int64_t)(Hql + Hkvl) * D;
  p.o = static_cast<const __bf16*>(o);
  p.dout = static_cast<const __bf16*>(dout);
  p.lse = lse;
  char* ws = static_cast<char*>(workspace);
  p.delta = reinterpret_cast<float*>(ws);
  p.lse2 = reinterpret_cast<float*>(ws + stat_bytes(B, S, Hql));
  p.ws_counters = reinterpret_cast<unsigned int*>(ws + 2 * stat_bytes(B, S, Hql));
  p.ds = nullptr;
  return ie::launch_bwd(p, D, IE_BWD_ALL, static_cast<hipStream_t>(stream));
}

int ie_attn_set_tile_rows(int32_t rows) {
  if (rows != 0 && rows != 128 && rows != 256) return IE_ERR_UNSUPPORTED;
  return ie::tile_rows_setting.exchange(rows, std::memory_order_relaxed);
}

const char* ie_attn_strerror(int code) {
  switch (code) {
    case IE_OK: return "success";
    case IE_ERR_NULL: return "a required pointer is NULL";
    case IE_ERR_SHAPE: return "invalid shape (sizes must be positive, Hq % Hkv == 0, packed input needs B == 1 and num_docs >= 1)";
    case IE_ERR_UNSUPPORTED: return "unsupported configuration (D must be 64 or 128, scale finite and > 0, causal 0 or 1; phase and path flags valid for the shape)";
    case IE_ERR_WORKSPACE: return "workspace missing, not 256-byte aligned, or too small";
    case IE_ERR_HIP: return "a HIP runtime call failed";
    case IE_ERR_ALIGN: return "a pointer is not 16-byte aligned";
    case IE_ERR_BUSY: return "every work-queue slot of the forward kernel is in flight or held by a captured graph";
    default: return "unknown ie_attn status";
  }
}

const char* ie_attn_last_hip_error(void) { return g_hip_error; }

}  // extern "C"
