// Measures what the bf16 matrix cores of this GPU sustain, as the denominator's reality check:
// a register-only loop of v_mfma_f32_32x32x16_bf16 (and, for comparison, of the 16x16x32 shape at the same
// FLOP per clock) with no memory, no LDS, no VALU work, four
// independent accumulators per wave, one wave per SIMD on every CU, run for a few seconds so
// that power management has settled.  Two operand regimes: small integers that never change
// (little switching activity), and N(0,1)-like values cycling through 8 register sets so that
// consecutive MFMAs see different inputs, as in a real contraction.
//
// Prints TFLOP/s and the clock that figure implies at 1024 FLOP/clk/SIMD x 4 SIMD x 256 CU,
// and - from the shader cycle counter and the constant 100 MHz counter read inside the kernel -
// how many shader cycles one MFMA took (32 = the pipe never idles) and the shader clock the
// kernel actually ran at: the two ways a power limit can show.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                          \
  do {                                                                                 \
    hipError_t e = (x);                                                                \
    if (e != hipSuccess) {                                                             \
      std::printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__);        \
      std::exit(1);                                                                    \
    }                                                                                  \
  } while (0)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ float pseudo_normal(unsigned& h) {  // sum of three uniforms, unit-ish variance
  float s = 0.f;
  for (int i = 0; i < 3; ++i) {
    h = h * 1664525u + 1013904223u;
    s += (h >> 8) * (1.0f / 16777216.0f);
  }
  return (s - 1.5f) * 2.0f;
}

// HOLD: how many consecutive MFMAs see the same A operand (1: every MFMA gets a new A and a new B; 4: A changes
// every fourth MFMA, as when one fragment feeds a row of output blocks; 0: A and B never change)
template <int NSET, bool RANDOM, bool SMALL, int HOLD = 1>
__global__ __launch_bounds__(256) void mfma_loop(float* out, unsigned long long* ticks, int iters) {
  const int tid = threadIdx.x;
  const unsigned long long c0 = __builtin_readcyclecounter(), w0 = wall_clock64();
  unsigned h = tid * 2654435761u + blockIdx.x * 40503u + 12345u;
  bf16x8 a[NSET], b[NSET];
  for (int i = 0; i < NSET; ++i)
    for (int t = 0; t < 8; ++t) {
      a[i][t] = RANDOM ? (__bf16)pseudo_normal(h) : (__bf16)(float)((tid * 7 + t) % 5 - 2);
      b[i][t] = RANDOM ? (__bf16)pseudo_normal(h) : (__bf16)(float)((tid + t) % 3 - 1);
    }
  float s = 0.f;
  if constexpr (SMALL) {   // 16x16x32: half the FLOP per instruction, so two per 32x32x16
    f32x4 c[8];
    for (int i = 0; i < 8; ++i)
      for (int r = 0; r < 4; ++r) c[i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int u = 0; u < 32; ++u)
        c[u & 7] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u % NSET], b[(u / 8 + u) % NSET], c[u & 7], 0, 0, 0);
    }
    for (int i = 0; i < 8; ++i)
      for (int r = 0; r < 4; ++r) s += c[i][r];
  } else {
    f32x16 c[4];
    for (int i = 0; i < 4; ++i)
      for (int r = 0; r < 16; ++r) c[i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int u = 0; u < 16; ++u)
        c[u & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[HOLD == 0 ? 0 : HOLD == 1 ? u % NSET : (u / HOLD) % NSET],
                                                           b[HOLD == 0 ? 0 : (u / 4 + u) % NSET], c[u & 3], 0, 0, 0);
    }
    for (int i = 0; i < 4; ++i)
      for (int r = 0; r < 16; ++r) s += c[i][r];
  }
  out[blockIdx.x * 256 + tid] = s;
  if (tid == 0) {
    ticks[2 * blockIdx.x] = __builtin_readcyclecounter() - c0;
    ticks[2 * blockIdx.x + 1] = wall_clock64() - w0;
  }
}

template <int NSET, bool RANDOM, bool SMALL = false, int HOLD = 1>
void run(float* out, unsigned long long* ticks, int cus, const char* name, double seconds) {
  const int iters = 20000;  // 16 MFMAs of 32768 FLOP per trip and wave
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  float ms = 0.f;
  const auto t0 = std::chrono::steady_clock::now();
  double elapsed = 0.0;
  while (elapsed < seconds) {
    CK(hipEventRecord(e0));
    mfma_loop<NSET, RANDOM, SMALL, HOLD><<<cus, 256>>>(out, ticks, iters);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    CK(hipEventElapsedTime(&ms, e0, e1));
    elapsed = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
  }
  const double flop = (double)cus * 4 * iters * 16 * 32768.0;
  const double tflops = flop / (ms * 1e-3) / 1e12;
  const double ghz = tflops * 1e12 / ((double)cus * 4 * 1024.0) / 1e9;
  std::printf("%-52s %8.1f TFLOP/s after %.1f s  (= %.2f GHz at 1024 FLOP/clk/SIMD)\n", name, tflops, elapsed, ghz);
  unsigned long long* h = (unsigned long long*)std::malloc((size_t)cus * 16);
  CK(hipMemcpy(h, ticks, (size_t)cus * 16, hipMemcpyDeviceToHost));
  double cyc = 0, wall = 0;
  for (int i = 0; i < cus; ++i) { cyc += (double)h[2 * i]; wall += (double)h[2 * i + 1]; }
  std::free(h);
  std::printf("%-52s %8.2f shader cycles per 32768 FLOP of MFMA, shader clock %.3f GHz (last launch, mean over workgroups)\n", "",
              cyc / cus / ((double)iters * 16), cyc / wall * 0.1);
}

int main(int argc, char** argv) {
  const double seconds = argc > 1 ? std::atof(argv[1]) : 3.0;
  hipDeviceProp_t prop;
  CK(hipGetDeviceProperties(&prop, 0));
  std::printf("device: %s, %d CUs, clock rate %.2f GHz\n", prop.gcnArchName, prop.multiProcessorCount, prop.clockRate / 1e6);
  float* out;
  CK(hipMalloc(&out, (size_t)prop.multiProcessorCount * 256 * sizeof(float)));
  unsigned long long* ticks;
  CK(hipMalloc(&ticks, (size_t)prop.multiProcessorCount * 16));
  run<1, false>(out, ticks, prop.multiProcessorCount, "32x32x16 bf16, constant small-integer operands", seconds);
  run<8, true>(out, ticks, prop.multiProcessorCount, "32x32x16 bf16, N(0,1) operands, 8 sets cycled", seconds);
  run<8, true, false, 4>(out, ticks, prop.multiProcessorCount, "32x32x16 bf16, N(0,1), A held for 4 MFMAs", seconds);
  run<8, true, false, 0>(out, ticks, prop.multiProcessorCount, "32x32x16 bf16, N(0,1), A and B never change", seconds);
  run<8, true, true>(out, ticks, prop.multiProcessorCount, "16x16x32 bf16, N(0,1) operands, 8 sets cycled", seconds);
  CK(hipFree(ticks));
  CK(hipFree(out));
  return 0;
}
