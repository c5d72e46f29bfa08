// Measurement aid for the benchmark, not part of the library: the rate at which this board
// sustains back-to-back bf16 32x32x16 MFMAs with NOTHING else going on, for all-zero, all-one
// and random operands.  The board holds a power limit by lowering the shader clock, and MFMA
// power depends on how many operand bits toggle, so the sustained rate on random data is well
// below the nominal peak (256 CUs x 4 SIMDs x 1024 flop/cycle x 2.4 GHz).  The benchmark prints
// this figure beside the attention kernel's so that both fractions can be read.
//
// Prints one line:  zeros <TFLOP/s> <MHz>  ones <TFLOP/s> <MHz>  random <TFLOP/s> <MHz>
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

#define CK(x)                                                                   \
  do {                                                                          \
    hipError_t e_ = (x);                                                        \
    if (e_ != hipSuccess) {                                                     \
      std::fprintf(stderr, "mfma_ceiling: %s (line %d)\n", hipGetErrorString(e_), __LINE__); \
      std::exit(1);                                                             \
    }                                                                           \
  } while (0)

// 8 waves per workgroup = 2 per SIMD, as in the attention kernel; 8 independent MFMAs per
// iteration on 4 accumulators, operands fixed in registers
__global__ __launch_bounds__(512) void mfma_loop(const bf16x8* __restrict__ in, float* __restrict__ out,
                                                 uint64_t* __restrict__ clk, int iters) {
  bf16x8 a[8], b[8];
  for (int i = 0; i < 8; ++i) {
    a[i] = in[threadIdx.x * 16 + i];
    b[i] = in[threadIdx.x * 16 + 8 + i];
  }
  f32x16 c[4];
  for (int n = 0; n < 4; ++n)
    for (int r = 0; r < 16; ++r) c[n][r] = 0.f;
  const uint64_t t0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) c[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[i], c[i & 3], 0, 0, 0);
    if ((it & 63) == 63)   // keep the accumulators bounded
      for (int n = 0; n < 4; ++n)
        for (int r = 0; r < 16; ++r) c[n][r] *= 1e-3f;
  }
  const uint64_t t1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  float s = 0;
  for (int n = 0; n < 4; ++n)
    for (int r = 0; r < 16; ++r) s += c[n][r];
  out[blockIdx.x * 512 + threadIdx.x] = s;
  if (blockIdx.x == 5 && threadIdx.x == 0) {
    clk[0] = t1 - t0;
    clk[1] = r1 - r0;
  }
}

int main(int argc, char** argv) {
  const int iters = argc > 1 ? std::atoi(argv[1]) : 60000;   // ~15 ms per mode: long enough for the clock to settle
  hipDeviceProp_t prop;
  CK(hipGetDeviceProperties(&prop, 0));
  const int cus = prop.multiProcessorCount;
  std::vector<uint16_t> h(512 * 16 * 8);
  bf16x8* in;
  float* out;
  uint64_t* clk;
  CK(hipMalloc(&in, h.size() * 2));
  CK(hipMalloc(&out, (size_t)cus * 512 * 4));
  CK(hipMalloc(&clk, 16));
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  const char* names[3] = {"zeros", "ones", "random"};
  for (int mode = 0; mode < 3; ++mode) {
    std::srand(1);
    for (auto& x : h) {
      if (mode == 0) x = 0;
      else if (mode == 1) x = 0x3F80;   // 1.0
      else {                            // uniform in [-2, 2], truncated to bf16
        const float f = ((std::rand() % 2001) - 1000) / 500.0f;
        uint32_t u;
        std::memcpy(&u, &f, 4);
        x = (uint16_t)(u >> 16);
      }
    }
    CK(hipMemcpy(in, h.data(), h.size() * 2, hipMemcpyHostToDevice));
    mfma_loop<<<cus, 512>>>(in, out, clk, iters / 30);   // warm-up
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    mfma_loop<<<cus, 512>>>(in, out, clk, iters);
    CK(hipEventRecord(e1));
    CK(hipDeviceSynchronize());
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    uint64_t c[2];
    CK(hipMemcpy(c, clk, 16, hipMemcpyDeviceToHost));
    const double flop = (double)cus * 8 * iters * 8 * 32768.0;
    // both counters are read by the same wave around the loop: their ratio times the 100 MHz
    // reference clock is the shader clock during the loop
    std::printf("%s %.1f %.0f  ", names[mode], flop / (ms * 1e-3) / 1e12, (double)c[0] / (double)c[1] * 100.0);
  }
  std::printf("\n");
  return 0;
}
