// What one wave can issue in the shadow of its MFMAs, measured in shader cycles on one CU.
//
// The attention kernels interleave v_mfma_f32_32x32x16_bf16 (32 cycles of matrix pipe each) with
// the softmax arithmetic, LDS reads and global->LDS copies.  This probe times "slots" of one
// MFMA followed by a fixed group of other instructions, for 1 to 4 waves per SIMD running the
// same stream, with the shader cycle counter read inside the kernel (so the result does not
// depend on the clock the power management happens to pick):
//   - how many plain VALU instructions / v_exp_f32 fit behind one MFMA of the same wave,
//   - what LDS reads add,
//   - what one global_load_lds_dwordx4 (the asynchronous copy) costs the wave that issues it.
// All operands are small constants: this measures issue, not power.
//
// Build: hipcc --offload-arch=gfx950 -O3 -o issue_cost_probe issue_cost_probe.hip   (build.py does it)
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                   \
  do {                                                                          \
    hipError_t e = (x);                                                         \
    if (e != hipSuccess) {                                                      \
      std::printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__); \
      std::exit(1);                                                             \
    }                                                                           \
  } while (0)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define REP4(x) x x x x
#define REP16(x) REP4(x) REP4(x) REP4(x) REP4(x)
// operands: %0-%3 accumulators, %4-%7 floats, %8/%9 LDS results, %10/%11 MFMA A/B, %12 LDS address
#define SLOT(acc) "v_mfma_f32_32x32x16_bf16 " acc ", %10, %11, " acc "\n"
#define BODY(n) REP4(SLOT("%0") n SLOT("%1") n SLOT("%2") n SLOT("%3") n)
#define F1 "v_fma_f32 %4, %4, %6, %7\n"
#define E1 "v_exp_f32 %5, %6\n"
#define SOFTMAX4 "v_fma_f32 %4, %5, %6, %7\n v_exp_f32 %4, %4\n v_add_f32 %5, %5, %6\n v_cvt_pk_bf16_f32 %7, %6, %4\n"
#define LDS2 "ds_read_b64 %8, %12\n ds_read_b64 %9, %12 offset:512\n"
#define OPS                                                                                                         \
  : "+v"(c0), "+v"(c1), "+v"(c2), "+v"(c3), "+v"(v0), "+v"(v1), "+v"(v2), "+v"(v3), "=v"(d0), "=v"(d1)               \
  : "v"(a), "v"(b), "v"(ldsaddr)
#define LOOP(x) \
  for (int it = 0; it < iters; ++it) asm volatile(x "s_waitcnt lgkmcnt(0)\n" OPS);

template <int MODE>
__global__ __launch_bounds__(1024) void slots(uint64_t* out, int iters) {
  __shared__ double lbuf[2048];
  const int tid = threadIdx.x, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  lbuf[tid] = tid;
  lbuf[tid + 1024] = tid;
  bf16x8 a, b;
  for (int t = 0; t < 8; ++t) { a[t] = (__bf16)(float)((tid * 7 + t) % 5 - 2); b[t] = (__bf16)(float)((tid + t) % 3 - 1); }
  f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  float v0 = tid * 0.001f, v1 = 1.f + v0, v2 = 2.f + v0, v3 = 3.f + v0;
  double d0 = 0, d1 = 0;
  const uint32_t ldsaddr = (uint32_t)(uintptr_t)lbuf + (tid & 63) * 8;
  __syncthreads();
  const uint64_t t0 = __builtin_readcyclecounter();
  if (MODE == 0) LOOP(BODY(""))
  if (MODE == 1) LOOP(BODY(F1 F1 F1))
  if (MODE == 2) LOOP(BODY(F1 F1 F1 F1 F1))
  if (MODE == 3) LOOP(BODY(F1 F1 F1 F1 F1 F1))
  if (MODE == 4) LOOP(BODY(F1 F1 F1 F1 F1 F1 F1 F1))
  if (MODE == 5) LOOP(BODY(E1 E1 E1))
  if (MODE == 6) LOOP(BODY(SOFTMAX4))
  if (MODE == 7) LOOP(BODY(SOFTMAX4 LDS2))
  if (MODE == 8) LOOP(BODY(SOFTMAX4 F1 F1 E1))
  const uint64_t t1 = __builtin_readcyclecounter();
  float s = v0 + v1 + v2 + v3 + (float)d0 + (float)d1;
  for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
  if ((tid & 63) == 0) out[wv] = t1 - t0;
  if (s == 12345.678f) out[0] = 0;
}

extern __shared__ __attribute__((aligned(16))) char smem[];

// 16 MFMAs per iteration with NC asynchronous copies of 1 KiB spread evenly between them.
template <int NC>
__global__ __launch_bounds__(256) void copies(uint64_t* out, const char* src, int iters) {
  const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  bf16x8 a, b;
  for (int t = 0; t < 8; ++t) { a[t] = (__bf16)(float)((tid * 7 + t) % 5 - 2); b[t] = (__bf16)(float)((tid + t) % 3 - 1); }
  f32x16 c[4] = {};
  const uint32_t lds = (uint32_t)(uintptr_t)smem + wv * 16384;
  const uint32_t voff = lane * 16;
  __syncthreads();
  const uint64_t t0 = __builtin_readcyclecounter();
  for (int it = 0; it < iters; ++it) {
    const char* g = src + (size_t)wv * (1 << 20) + (size_t)(it & 255) * 4096;
#pragma unroll
    for (int sl = 0; sl < 16; ++sl) {
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c[sl & 3]) : "v"(a), "v"(b));
      if (NC > 0 && sl % (16 / (NC > 0 ? NC : 1)) == 0) {
        const int k = sl / (16 / (NC > 0 ? NC : 1));
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(g + k * 1024), "s"(lds + k * 1024)
                     : "memory");
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  const uint64_t t1 = __builtin_readcyclecounter();
  float s = smem[tid];
  for (int i = 0; i < 4; ++i)
    for (int q = 0; q < 16; ++q) s += c[i][q];
  if (lane == 0) out[wv] = t1 - t0;
  if (s == 12345.678f) out[0] = 0;
}

template <int MODE>
void run_slots(const char* name, uint64_t* out) {
  const int iters = 2000;
  std::printf("%-44s", name);
  for (int threads = 256; threads <= 1024; threads += 256) {
    slots<MODE><<<1, threads>>>(out, iters);
    CK(hipDeviceSynchronize());
    slots<MODE><<<1, threads>>>(out, iters);
    CK(hipDeviceSynchronize());
    uint64_t h[16];
    CK(hipMemcpy(h, out, sizeof(h), hipMemcpyDeviceToHost));
    const int per_simd = threads / 256;
    // the last wave to finish bounds the SIMD; it ran 16 slots per iteration, as did its per_simd - 1 neighbours
    uint64_t worst = 0;
    for (int w = 0; w < threads / 64; ++w) worst = h[w] > worst ? h[w] : worst;
    std::printf("  %6.1f", (double)worst / iters / 16 / per_simd);
  }
  std::printf("\n");
}

template <int NC>
void run_copies(uint64_t* out, const char* src, double base) {
  const int iters = 2000;
  CK(hipFuncSetAttribute((const void*)copies<NC>, hipFuncAttributeMaxDynamicSharedMemorySize, 65536));
  copies<NC><<<1, 256, 65536>>>(out, src, iters);
  CK(hipDeviceSynchronize());
  copies<NC><<<1, 256, 65536>>>(out, src, iters);
  CK(hipDeviceSynchronize());
  uint64_t h[4];
  CK(hipMemcpy(h, out, sizeof(h), hipMemcpyDeviceToHost));
  const double per_slot = (double)h[0] / iters / 16;
  std::printf("16 MFMAs + %d global_load_lds_dwordx4: %6.2f cycles per MFMA", NC, per_slot);
  if (NC > 0) std::printf("  (= %5.1f cycles per copy instruction)", (per_slot - base) * 16 / NC);
  std::printf("\n");
}

int main() {
  uint64_t* out;
  CK(hipMalloc(&out, 16 * sizeof(uint64_t)));
  char* src;
  CK(hipMalloc(&src, (size_t)8 << 20));
  CK(hipMemset(src, 1, (size_t)8 << 20));
  std::printf("shader cycles per MFMA of the SIMD (32 = matrix pipe never idles), by waves per SIMD\n");
  std::printf("%-44s  %6s  %6s  %6s  %6s\n", "slot = one MFMA followed by", "1", "2", "3", "4");
  run_slots<0>("nothing", out);
  run_slots<1>("3 v_fma_f32", out);
  run_slots<2>("5 v_fma_f32", out);
  run_slots<3>("6 v_fma_f32", out);
  run_slots<4>("8 v_fma_f32", out);
  run_slots<5>("3 v_exp_f32", out);
  run_slots<6>("fma, exp, add, cvt_pk", out);
  run_slots<7>("fma, exp, add, cvt_pk + 2 ds_read_b64", out);
  run_slots<8>("fma, exp, add, cvt_pk, fma, fma, exp", out);
  std::printf("\none workgroup of 4 waves (one per SIMD), every wave issues the copies:\n");
  run_copies<0>(out, src, 0);
  uint64_t h0;
  CK(hipMemcpy(&h0, out, 8, hipMemcpyDeviceToHost));
  const double base = (double)h0 / 2000 / 16;
  run_copies<1>(out, src, base);
  run_copies<2>(out, src, base);
  run_copies<4>(out, src, base);
  CK(hipFree(src));
  CK(hipFree(out));
  return 0;
}
