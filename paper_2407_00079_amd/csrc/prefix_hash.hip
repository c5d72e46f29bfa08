// Prefix block keys and longest prefix match for gfx950 (paper Algorithm 1: PrefixHash and
// FindBestPrefixMatch; Figure "KVCache pool": a block's hash value is determined by its own hash
// and by its prefix).  The paper fixes the block size (512 tokens), not the hash; the one used
// here is stated in include/mc.h.  Integer work, bit-exact against the CPU oracle.
//
//   digest kernel  one wave per block: every lane mixes its tokens (position-salted), the 64
//                  partial sums are added across the wave, lane 0 finalises.  Blocks are
//                  independent, so a batch of long prompts fills the GPU.
//   chain kernel   one wave per request walks its digests in order and turns them into keys in
//                  place (the only sequential part: one mix per block, on the scalar unit).
//   match kernel   one workgroup per (instance, request): thread t looks keys t, t + 256, ... up
//                  in the instance's ascending key array by bisection; the smallest index that
//                  misses is the prefix length.
//   best kernel    one thread per request scans its row of prefix lengths.
#include "mc_internal.h"

namespace mc {
namespace {

__device__ __forceinline__ uint64_t mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

// Blocks of one request sit along blockIdx.x (four per workgroup, one wave each), requests along
// blockIdx.y: no search for the owner of a block, and the offset tables are read by scalar loads.
__global__ __launch_bounds__(256) void prefix_digest_kernel(const int32_t* __restrict__ tokens,
                                                            const int64_t* __restrict__ tok_off,
                                                            const int64_t* __restrict__ key_off, int batch,
                                                            int block_tokens, uint64_t* __restrict__ keys) {
  const int lane = threadIdx.x & 63;
  const int64_t b = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  for (int r = blockIdx.y; r < batch; r += gridDim.y) {
    const int64_t k0 = key_off[r];
    if (b >= key_off[r + 1] - k0) continue;              // whole wave skips together
    const int64_t t0 = tok_off[r];
    const int64_t left = tok_off[r + 1] - t0 - b * block_tokens;
    const int nb = left < block_tokens ? (int)left : block_tokens;
    const int32_t* t = tokens + t0 + b * block_tokens;
    uint64_t sum = 0;
    int j = lane;
    for (; j + 7 * 64 < nb; j += 8 * 64) {                // eight loads in flight per lane
      int32_t v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = t[j + 64 * u];
#pragma unroll
      for (int u = 0; u < 8; ++u) sum += mix64((uint64_t)(uint32_t)v[u] + ((uint64_t)(j + 64 * u) << 32));
    }
    for (; j < nb; j += 64) sum += mix64((uint64_t)(uint32_t)t[j] + ((uint64_t)j << 32));
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
      const uint32_t lo = __shfl_xor((uint32_t)sum, d, 64), hi = __shfl_xor((uint32_t)(sum >> 32), d, 64);
      sum += ((uint64_t)hi << 32) | lo;
    }
    if (lane == 0) keys[k0 + b] = mix64(sum + (uint64_t)nb);
  }
}

// One wave per request.  The chain itself is sequential, but its loads and stores need not be:
// the wave reads 64 digests at once, walks them lane by lane with wave-uniform (scalar unit)
// arithmetic, each lane keeping the key of its own block, and writes the 64 keys back at once.
__global__ __launch_bounds__(64) void prefix_chain_kernel(const int64_t* __restrict__ key_off, int batch,
                                                          uint64_t* __restrict__ keys) {
  const int lane = threadIdx.x;
  for (int r = blockIdx.x; r < batch; r += gridDim.x) {
    const int64_t k0 = key_off[r], nk = key_off[r + 1] - k0;
    uint64_t prev = 0;
    for (int64_t base = 0; base < nk; base += 64) {
      const int64_t i = base + lane;
      const uint64_t digest = i < nk ? keys[k0 + i] : 0;
      const int m = nk - base < 64 ? (int)(nk - base) : 64;
      uint64_t mine = 0;
      for (int j = 0; j < m; ++j) {
        const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)digest, j);
        const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(digest >> 32), j);
        const uint64_t d = ((uint64_t)hi << 32) | lo;
        const uint64_t salt = base + j == 0 ? 0x243F6A8885A308D3ull
                                            : ((prev << 23) | (prev >> 41)) * 0x9E3779B97F4A7C15ull;
        prev = mix64(d ^ salt);
        if (lane == j) mine = prev;
      }
      if (i < nk) keys[k0 + i] = mine;
    }
  }
}

__global__ __launch_bounds__(256) void prefix_match_kernel(const uint64_t* __restrict__ keys,
                                                           const int64_t* __restrict__ key_off,
                                                           const uint64_t* __restrict__ cache_keys,
                                                           const int64_t* __restrict__ cache_off, int n_inst,
                                                           int32_t* __restrict__ prefix_len) {
  __shared__ int first_miss;
  const int inst = blockIdx.x, r = blockIdx.y;
  const int64_t k0 = key_off[r], nk = key_off[r + 1] - k0;
  const uint64_t* c = cache_keys + cache_off[inst];
  const int64_t nc = cache_off[inst + 1] - cache_off[inst];
  if (threadIdx.x == 0) first_miss = (int)nk;
  __syncthreads();
  for (int64_t base = 0; base < nk; base += 256) {
    const int64_t i = base + threadIdx.x;
    if (i < nk) {
      const uint64_t key = keys[k0 + i];
      int64_t lo = 0, hi = nc;                           // first element >= key
      while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (c[mid] < key) lo = mid + 1; else hi = mid;
      }
      if (!(lo < nc && c[lo] == key)) atomicMin(&first_miss, (int)i);
    }
    __syncthreads();
    if (first_miss < base + 256) break;                  // uniform: everyone reads the same value after the barrier
    __syncthreads();
  }
  if (threadIdx.x == 0) prefix_len[(int64_t)r * n_inst + inst] = first_miss;
}

__global__ __launch_bounds__(64) void prefix_best_kernel(const int32_t* __restrict__ prefix_len, int batch, int n_inst,
                                                         int32_t* __restrict__ best_len,
                                                         int32_t* __restrict__ best_inst) {
  const int r = blockIdx.x * 64 + threadIdx.x;
  if (r >= batch) return;
  int32_t bl = 0, bi = n_inst > 0 ? 0 : -1;
  for (int i = 0; i < n_inst; ++i) {
    const int32_t l = prefix_len[(int64_t)r * n_inst + i];
    if (l > bl) {
      bl = l;
      bi = i;
    }
  }
  best_len[r] = bl;
  best_inst[r] = bi;
}

}  // namespace

hipError_t launch_prefix_hash(const int32_t* tokens, const int64_t* tok_off, const int64_t* key_off, int batch,
                              int block_tokens, int64_t max_blocks, uint64_t* keys, hipStream_t stream) {
  (void)hipGetLastError();
  const unsigned req_rows = batch < 65535 ? (unsigned)batch : 65535u;   // the kernels stride over the rest
  prefix_digest_kernel<<<dim3((unsigned)((max_blocks + 3) / 4), req_rows), 256, 0, stream>>>(
      tokens, tok_off, key_off, batch, block_tokens, keys);
  prefix_chain_kernel<<<req_rows, 64, 0, stream>>>(key_off, batch, keys);
  return hipGetLastError();
}

hipError_t launch_prefix_match(const uint64_t* keys, const int64_t* key_off, int batch, const uint64_t* cache_keys,
                               const int64_t* cache_off, int n_inst, int32_t* prefix_len, int32_t* best_len,
                               int32_t* best_inst, hipStream_t stream) {
  (void)hipGetLastError();
  if (n_inst > 0)
    prefix_match_kernel<<<dim3((unsigned)n_inst, (unsigned)batch), 256, 0, stream>>>(keys, key_off, cache_keys,
                                                                                     cache_off, n_inst, prefix_len);
  prefix_best_kernel<<<(unsigned)((batch + 63) / 64), 64, 0, stream>>>(prefix_len, batch, n_inst, best_len, best_inst);
  return hipGetLastError();
}

}  // namespace mc
