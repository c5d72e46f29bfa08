// Measurement aids of the benchmark, not part of the library.  What this board sustains with
// NOTHING else going on, so that the kernels' figures can be read against it:
//
//   bench_probes mfma [iters]
//       back-to-back bf16 MFMAs on all-zero, all-one and random (N(0,1)) operands, for the
//       32x32x16 tile and for the 16x16x32 tile in the accumulator pattern of the attention
//       kernel (each operand fragment feeds two MFMAs).  The board holds a power limit by
//       lowering the shader clock and MFMA power depends on operand bit activity and on the
//       tile shape, so the sustained rate on random data is well below the nominal peak
//       (256 CUs x 4 SIMDs x 1024 flop/cycle x 2.4 GHz = 2516.6 TFLOP/s).
//   bench_probes copy
//       the page copy of one configuration-5 layer (2048 pages of 32 KiB for K and for V,
//       scattered source, contiguous destination) with the library kernel's shape, beside the
//       read-only and the write-only half of the same access pattern, and the copy at 1/4x ..
//       2x the size (fixed cost per launch and rate of the steady state by a straight-line fit).
//   bench_probes copy-sweep
//       the same copy in every variant that was tried (slice size, threads, loads in flight,
//       cache-policy bits, K and V in one or two workgroups, persistent and pipelined grids).
//
// `mfma` and `copy` print one JSON object; `copy-sweep` prints a table.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <numeric>
#include <random>
#include <string>
#include <vector>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define CK(x)                                                                                  \
  do {                                                                                         \
    hipError_t e_ = (x);                                                                       \
    if (e_ != hipSuccess) {                                                                    \
      std::fprintf(stderr, "bench_probes: %s (line %d)\n", hipGetErrorString(e_), __LINE__);   \
      std::exit(1);                                                                            \
    }                                                                                          \
  } while (0)

// ------------------------------------------------------------------------------------------
// MFMA rates.  8 waves per workgroup = 2 per SIMD, one workgroup per CU, operands in registers.
// ------------------------------------------------------------------------------------------
// 32x32x16: 8 MFMAs into one accumulator (a score block) + 8 into 4 accumulators (P V), as the fp32-style kernel did
__global__ __launch_bounds__(512) void mfma_32x32x16(const bf16x8* __restrict__ in, float* __restrict__ out,
                                                     uint64_t* __restrict__ ticks, int iters) {
  bf16x8 a[8], b[8];
  for (int i = 0; i < 8; ++i) {
    a[i] = in[threadIdx.x * 16 + i];
    b[i] = in[threadIdx.x * 16 + 8 + i];
  }
  f32x16 s, o[4];
  for (int r = 0; r < 16; ++r) {
    s[r] = 0.f;
    for (int n = 0; n < 4; ++n) o[n][r] = 0.f;
  }
  const uint64_t t0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[i], s, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[i], a[i >> 2], o[i & 3], 0, 0, 0);
    if ((it & 63) == 63)   // keep the accumulators bounded
      for (int r = 0; r < 16; ++r) {
        s[r] *= 1e-3f;
        for (int n = 0; n < 4; ++n) o[n][r] *= 1e-3f;
      }
  }
  const uint64_t t1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  float acc = 0;
  for (int r = 0; r < 16; ++r) {
    acc += s[r];
    for (int n = 0; n < 4; ++n) acc += o[n][r];
  }
  out[blockIdx.x * 512 + threadIdx.x] = acc;
  if (blockIdx.x == 5 && threadIdx.x == 0) {
    ticks[0] = t1 - t0;
    ticks[1] = r1 - r0;
  }
}
// 16x16x32: 16 score MFMAs (2 key tiles x 2 row tiles x 4 steps) + 16 P V MFMAs (8 column tiles x 2 row tiles),
// every A fragment used by two consecutive MFMAs, as attn_prefill_bf16.hip issues them
__global__ __launch_bounds__(512) void mfma_16x16x32(const bf16x8* __restrict__ in, float* __restrict__ out,
                                                     uint64_t* __restrict__ ticks, int iters) {
  bf16x8 a[8], b[8];
  for (int i = 0; i < 8; ++i) {
    a[i] = in[threadIdx.x * 16 + i];
    b[i] = in[threadIdx.x * 16 + 8 + i];
  }
  f32x4 s[4], o[16];
  for (int r = 0; r < 4; ++r) {
    for (int n = 0; n < 4; ++n) s[n][r] = 0.f;
    for (int n = 0; n < 16; ++n) o[n][r] = 0.f;
  }
  const uint64_t t0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      s[(i & 1) * 2 + 0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[i >> 1], s[(i & 1) * 2 + 0], 0, 0, 0);
      s[(i & 1) * 2 + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[4 + (i >> 1)], s[(i & 1) * 2 + 1], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      o[2 * i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[i], a[0], o[2 * i], 0, 0, 0);
      o[2 * i + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[i], a[1], o[2 * i + 1], 0, 0, 0);
    }
    if ((it & 63) == 63)
      for (int r = 0; r < 4; ++r) {
        for (int n = 0; n < 4; ++n) s[n][r] *= 1e-3f;
        for (int n = 0; n < 16; ++n) o[n][r] *= 1e-3f;
      }
  }
  const uint64_t t1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  float acc = 0;
  for (int r = 0; r < 4; ++r) {
    for (int n = 0; n < 4; ++n) acc += s[n][r];
    for (int n = 0; n < 16; ++n) acc += o[n][r];
  }
  out[blockIdx.x * 512 + threadIdx.x] = acc;
  if (blockIdx.x == 5 && threadIdx.x == 0) {
    ticks[0] = t1 - t0;
    ticks[1] = r1 - r0;
  }
}

static uint16_t bf16_of(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  u += 0x7FFF + ((u >> 16) & 1);
  return (uint16_t)(u >> 16);
}

static int run_mfma(int iters) {
  hipDeviceProp_t prop;
  CK(hipGetDeviceProperties(&prop, 0));
  const int cus = prop.multiProcessorCount;
  std::vector<uint16_t> h(512 * 16 * 8);
  bf16x8* in;
  float* out;
  uint64_t* ticks;
  CK(hipMalloc(&in, h.size() * 2));
  CK(hipMalloc(&out, (size_t)cus * 512 * 4));
  CK(hipMalloc(&ticks, 16));
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  const char* data_names[3] = {"zeros", "ones", "random"};
  const char* shape_names[2] = {"32x32x16", "16x16x32"};
  std::printf("{");
  for (int shape = 0; shape < 2; ++shape) {
    std::printf("%s\"%s\": {", shape ? ", " : "", shape_names[shape]);
    for (int mode = 0; mode < 3; ++mode) {
      std::mt19937 gen(1);
      std::normal_distribution<float> nd(0.f, 1.f);
      for (auto& x : h) x = mode == 0 ? 0 : mode == 1 ? 0x3F80 : bf16_of(nd(gen));
      CK(hipMemcpy(in, h.data(), h.size() * 2, hipMemcpyHostToDevice));
      auto launch = [&](int n) {
        if (shape == 0) mfma_32x32x16<<<cus, 512>>>(in, out, ticks, n);
        else mfma_16x16x32<<<cus, 512>>>(in, out, ticks, n);
      };
      launch(iters / 4);   // warm-up: lets the clock settle
      CK(hipDeviceSynchronize());
      CK(hipEventRecord(e0));
      launch(iters);
      CK(hipEventRecord(e1));
      CK(hipDeviceSynchronize());
      float ms;
      CK(hipEventElapsedTime(&ms, e0, e1));
      uint64_t t[2];
      CK(hipMemcpy(t, ticks, 16, hipMemcpyDeviceToHost));
      const double flop = (double)cus * 8 * iters * 16 * 32768.0;   // both loops: 524288 flop per wave and iteration
      // both counters are read by the same wave around the loop: their ratio times the 100 MHz of the
      // constant clock is the rate of the cycle counter during the loop
      const double mhz = (double)t[0] / (double)t[1] * 100.0;
      std::printf("%s\"%s\": {\"tflops\": %.1f, \"shader_mhz\": %.0f}", mode ? ", " : "", data_names[mode],
                  flop / (ms * 1e-3) / 1e12, mhz);
    }
    std::printf("}");
  }
  std::printf("}\n");
  return 0;
}

// ------------------------------------------------------------------------------------------
// Page copies.  MODE 0 copy, 1 read only, 2 write only.  Scattered pages -> contiguous (pack shape).
// ------------------------------------------------------------------------------------------
template <int THREADS, int UNROLL, int MODE, bool NTL, bool NTS, bool KVX>
__global__ __launch_bounds__(THREADS) void copy_slice(const u32x4* __restrict__ ks, const u32x4* __restrict__ vs,
                                                      u32x4* __restrict__ kd, u32x4* __restrict__ vd,
                                                      const int32_t* __restrict__ ids, int64_t page_vecs, int slices,
                                                      u32x4* sink) {
  int bx = blockIdx.x, which = blockIdx.y;
  if (KVX) {   // K and V of a slice by neighbouring workgroups of one grid row
    which = bx & 1;
    bx >>= 1;
  }
  const int page = bx / slices, slice = bx - page * slices;
  const int64_t pool_page = ids[page];
  const u32x4* src = (which ? vs : ks) + pool_page * page_vecs;
  u32x4* dst = (which ? vd : kd) + (int64_t)page * page_vecs;
  const int64_t first = (int64_t)slice * THREADS * UNROLL + threadIdx.x;
  u32x4 v[UNROLL];
  if (MODE != 2) {
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) v[u] = NTL ? __builtin_nontemporal_load(src + first + u * THREADS) : src[first + u * THREADS];
  } else {
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) v[u] = u32x4{(uint32_t)bx, (uint32_t)threadIdx.x, (uint32_t)u, 7u};
  }
  if (MODE != 1) {
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      if (NTS) __builtin_nontemporal_store(v[u], dst + first + u * THREADS);
      else dst[first + u * THREADS] = v[u];
    }
  } else {
    u32x4 acc = v[0];
#pragma unroll
    for (int u = 1; u < UNROLL; ++u) acc ^= v[u];
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) sink[threadIdx.x] = acc;   // keeps the loads alive
  }
}
// persistent grid, software pipelined: the loads of a workgroup's next slice are issued before the stores of this one
template <int THREADS, int UNROLL>
__global__ __launch_bounds__(THREADS) void copy_pipelined(const u32x4* __restrict__ ks, const u32x4* __restrict__ vs,
                                                          u32x4* __restrict__ kd, u32x4* __restrict__ vd,
                                                          const int32_t* __restrict__ ids, int64_t page_vecs, int n_units,
                                                          int slices) {
  auto addr = [&](int unit, const u32x4*& src, u32x4*& dst) {
    const int which = unit & 1, rest = unit >> 1;
    const int page = rest / slices, slice = rest - page * slices;
    const int64_t first = (int64_t)slice * THREADS * UNROLL + threadIdx.x;
    src = (which ? vs : ks) + (int64_t)ids[page] * page_vecs + first;
    dst = (which ? vd : kd) + (int64_t)page * page_vecs + first;
  };
  int unit = blockIdx.x;
  if (unit >= n_units) return;
  const u32x4* src;
  u32x4* dst;
  addr(unit, src, dst);
  u32x4 v[UNROLL];
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) v[u] = __builtin_nontemporal_load(src + u * THREADS);
  for (;;) {
    const int next = unit + gridDim.x;
    u32x4 w[UNROLL];
    const u32x4* nsrc = src;
    u32x4* ndst = dst;
    const bool more = next < n_units;
    if (more) {
      addr(next, nsrc, ndst);
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) w[u] = __builtin_nontemporal_load(nsrc + u * THREADS);
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) __builtin_nontemporal_store(v[u], dst + u * THREADS);
    if (!more) break;
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) v[u] = w[u];
    unit = next;
    src = nsrc;
    dst = ndst;
  }
}
// two phases per workgroup: ALL loads of a unit (UNROLL KiB per wave) land before its first store is issued
template <int THREADS, int UNROLL>
__global__ __launch_bounds__(THREADS) void copy_two_phase(const u32x4* __restrict__ ks, const u32x4* __restrict__ vs,
                                                          u32x4* __restrict__ kd, u32x4* __restrict__ vd,
                                                          const int32_t* __restrict__ ids, int n, int parts) {
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * (THREADS / 64) + (threadIdx.x >> 6);
  const int n_waves = gridDim.x * (THREADS / 64);
  const int units = 2 * n * parts;
  for (int unit = wave; unit < units; unit += n_waves) {
    const int part = unit / (2 * n), t = unit - part * 2 * n;
    const int which = t >= n, page = which ? t - n : t;
    const int64_t page_vecs = (int64_t)parts * UNROLL * 64;
    const u32x4* src = (which ? vs : ks) + (int64_t)ids[page] * page_vecs + part * UNROLL * 64 + lane;
    u32x4* dst = (which ? vd : kd) + (int64_t)page * page_vecs + part * UNROLL * 64 + lane;
    u32x4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) v[u] = __builtin_nontemporal_load(src + u * 64);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) __builtin_nontemporal_store(v[u], dst + u * 64);
  }
}

struct CopyBench {
  static constexpr int kSets = 8;          // rotating buffer sets: 3 GiB in all, far beyond the 256 MiB last-level cache
  static constexpr int N = 4096;
  static constexpr int64_t pb = 32768, pv = pb / 16;
  std::vector<u32x4*> kp, vp, ko, vo;
  int32_t* ids = nullptr;
  u32x4* sink = nullptr;
  hipEvent_t a, b;
  CopyBench() : kp(kSets), vp(kSets), ko(kSets), vo(kSets) {
    for (int s = 0; s < kSets; ++s) {
      CK(hipMalloc(&kp[s], N * pb));
      CK(hipMalloc(&vp[s], N * pb));
      CK(hipMalloc(&ko[s], N * pb));
      CK(hipMalloc(&vo[s], N * pb));
      CK(hipMemset(kp[s], s + 1, N * pb));
      CK(hipMemset(vp[s], s + 7, N * pb));
    }
    CK(hipMalloc(&sink, 1024 * 16));
    std::vector<int32_t> h(N);
    std::iota(h.begin(), h.end(), 0);
    std::mt19937 g(20240705);
    std::shuffle(h.begin(), h.end(), g);
    CK(hipMalloc(&ids, N * 4));
    CK(hipMemcpy(ids, h.data(), N * 4, hipMemcpyHostToDevice));
    CK(hipEventCreate(&a));
    CK(hipEventCreate(&b));
  }
  // microseconds per launch: best of 3 runs of 80 back-to-back launches on rotating buffers
  template <class F>
  double time_us(F launch) {
    for (int i = 0; i < kSets; ++i) launch(i);
    CK(hipDeviceSynchronize());
    double best = 1e30;
    for (int trial = 0; trial < 3; ++trial) {
      CK(hipEventRecord(a));
      for (int i = 0; i < 80; ++i) launch(i % kSets);
      CK(hipEventRecord(b));
      CK(hipEventSynchronize(b));
      float ms;
      CK(hipEventElapsedTime(&ms, a, b));
      best = std::min(best, (double)ms * 1e3 / 80);
    }
    return best;
  }
  template <int T, int U, int MODE, bool NTL, bool NTS, bool KVX>
  double slice_us(int n) {
    return time_us([&](int s) {
      const int slices = pv / (T * U);
      dim3 grid(KVX ? n * slices * 2 : n * slices, KVX ? 1 : 2);
      copy_slice<T, U, MODE, NTL, NTS, KVX><<<grid, T>>>(kp[s], vp[s], ko[s], vo[s], ids, pv, slices, sink);
    });
  }
};

static int run_copy() {
  CopyBench cb;
  const int n = 2048;
  const double copy_bytes = 4.0 * n * cb.pb, half_bytes = 2.0 * n * cb.pb;
  const double t_copy = cb.slice_us<512, 1, 0, true, true, false>(n);
  const double t_read = cb.slice_us<512, 1, 1, true, true, false>(n);
  const double t_write = cb.slice_us<512, 1, 2, true, true, false>(n);
  // the same copy at other sizes: time = fixed + bytes / rate
  const int sizes[5] = {512, 1024, 2048, 3072, 4096};
  double t[5], sx = 0, sy = 0, sxx = 0, sxy = 0;
  for (int i = 0; i < 5; ++i) {
    t[i] = cb.slice_us<512, 1, 0, true, true, false>(sizes[i]);
    const double x = 4.0 * sizes[i] * cb.pb;
    sx += x, sy += t[i], sxx += x * x, sxy += x * t[i];
  }
  const double slope = (5 * sxy - sx * sy) / (5 * sxx - sx * sx), fixed = (sy - slope * sx) / 5;
  std::printf("{\"copy\": {\"us\": %.2f, \"GBs\": %.1f}, \"read_only\": {\"us\": %.2f, \"GBs\": %.1f}, "
              "\"write_only\": {\"us\": %.2f, \"GBs\": %.1f}, \"copy_by_size\": {",
              t_copy, copy_bytes / t_copy / 1e3, t_read, half_bytes / t_read / 1e3, t_write, half_bytes / t_write / 1e3);
  for (int i = 0; i < 5; ++i) std::printf("%s\"%d_pages\": %.2f", i ? ", " : "", sizes[i], t[i]);
  std::printf("}, \"fixed_us_per_launch\": %.2f, \"steady_state_GBs\": %.1f}\n", fixed, 1.0 / slope / 1e3);
  return 0;
}

static int run_copy_sweep() {
  CopyBench cb;
  const int n = 2048;
  const double CB = 4.0 * n * cb.pb, HB = 2.0 * n * cb.pb;
  auto row = [](const char* name, double us, double bytes) {
    std::printf("%-66s %7.2f us  %7.1f GB/s  %5.1f %% of 8 TB/s\n", name, us, bytes / us / 1e3, bytes / us / 1e3 / 80.0);
    std::fflush(stdout);
  };
  std::printf("# one configuration-5 layer: 2048 scattered pages of 32 KiB for K and for V -> contiguous; 80 launches back to\n"
              "# back on 8 rotating buffer sets (3 GiB), best of 3; T = threads per workgroup, U = 16-byte vectors per thread\n"
              "# (all loads of a thread are issued before its first store); nt = nontemporal\n");
  std::printf("--- copy, 268,435,456 B per launch: one workgroup per slice of T x U x 16 bytes\n");
#define SL(T, U, NTL, NTS, KVX, WHAT) row(WHAT, cb.slice_us<T, U, 0, NTL, NTS, KVX>(n), CB)
  SL(512, 1, true, true, false, "T=512 U=1 (8 KiB slices; the library's kernel)");
  SL(512, 1, true, true, true, "T=512 U=1, K and V slices in neighbouring workgroups");
  SL(512, 2, true, true, false, "T=512 U=2 (16 KiB)");
  SL(512, 4, true, true, false, "T=512 U=4 (whole 32 KiB page per workgroup)");
  SL(256, 1, true, true, false, "T=256 U=1 (4 KiB)");
  SL(256, 2, true, true, false, "T=256 U=2 (8 KiB)");
  SL(256, 4, true, true, false, "T=256 U=4 (16 KiB)");
  SL(256, 8, true, true, false, "T=256 U=8 (32 KiB)");
  SL(1024, 1, true, true, false, "T=1024 U=1 (16 KiB)");
  SL(1024, 2, true, true, false, "T=1024 U=2 (32 KiB)");
  SL(128, 4, true, true, false, "T=128 U=4 (8 KiB)");
  SL(64, 8, true, true, false, "T=64 U=8 (8 KiB, one wave)");
  SL(512, 1, false, true, false, "T=512 U=1, cached loads, nt stores");
  SL(512, 1, true, false, false, "T=512 U=1, nt loads, cached stores");
  SL(512, 1, false, false, false, "T=512 U=1, cached loads and stores");
  std::printf("--- copy, persistent grids\n");
#define PP(T, U, G) row("pipelined (next loads before these stores) T=" #T " U=" #U " grid=" #G, cb.time_us([&](int s) { \
    const int slices = cb.pv / (T * U); copy_pipelined<T, U><<<G, T>>>(cb.kp[s], cb.vp[s], cb.ko[s], cb.vo[s], cb.ids, cb.pv, n * 2 * slices, slices); }), CB)
  PP(256, 4, 2048);
  PP(512, 4, 512);
  PP(512, 1, 4096);
#define TP(T, U, G) row("two-phase (all loads land, then all stores) T=" #T " KiB/wave=" #U " grid=" #G, cb.time_us([&](int s) { \
    copy_two_phase<T, U><<<G, T>>>(cb.kp[s], cb.vp[s], cb.ko[s], cb.vo[s], cb.ids, n, 32 / U); }), CB)
  TP(1024, 16, 256);
  TP(512, 32, 512);
  TP(256, 16, 2048);
  TP(512, 8, 1024);
  std::printf("--- one direction only, 134,217,728 B per launch (T=512 U=1)\n");
  row("read only (scattered pages)", cb.slice_us<512, 1, 1, true, true, false>(n), HB);
  row("write only (contiguous)", cb.slice_us<512, 1, 2, true, true, false>(n), HB);
  row("read only, T=256 U=4", cb.slice_us<256, 4, 1, true, true, false>(n), HB);
  row("write only, T=256 U=4", cb.slice_us<256, 4, 2, true, true, false>(n), HB);
  std::printf("--- the library's shape at other sizes (time = fixed cost per launch + bytes / steady-state rate)\n");
  for (int pages : {128, 256, 512, 1024, 2048, 3072, 4096}) {
    char name[96];
    std::snprintf(name, sizeof name, "copy of %d pages", pages);
    row(name, cb.slice_us<512, 1, 0, true, true, false>(pages), 4.0 * pages * cb.pb);
  }
  std::printf("--- runtime\n");
  row("hipMemcpyDtoD of the same bytes, contiguous", cb.time_us([&](int s) {
        CK(hipMemcpyAsync(cb.ko[s], cb.kp[s], n * cb.pb, hipMemcpyDeviceToDevice, 0));
        CK(hipMemcpyAsync(cb.vo[s], cb.vp[s], n * cb.pb, hipMemcpyDeviceToDevice, 0));
      }), CB);
  return 0;
}

int main(int argc, char** argv) {
  const std::string mode = argc > 1 ? argv[1] : "mfma";
  if (mode == "mfma") return run_mfma(argc > 2 ? std::atoi(argv[2]) : 40000);
  if (mode == "copy") return run_copy();
  if (mode == "copy-sweep") return run_copy_sweep();
  std::fprintf(stderr, "usage: bench_probes mfma [iters] | copy | copy-sweep\n");
  return 2;
}
