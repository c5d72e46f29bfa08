// Prefix block keys and longest prefix match for gfx950 (paper Algorithm 1: PrefixHash and
// FindBestPrefixMatch; Figure "KVCache pool": a block's hash value is determined by its own hash
// and by its prefix).  The paper fixes the block size (512 tokens), not the hash; the one used
// here is stated in include/mc.h.  Integer work, bit-exact against the CPU oracle.
//
//   digest kernel  one wave per block: every lane mixes its tokens (position-salted), the 64
//                  partial sums are added across the wave, lane 0 finalises.  Blocks are
//                  independent, so a batch of long prompts fills the GPU.
//   chain kernel   one thread per request walks its digests in order and turns them into keys in
//                  place (the only sequential part: one mix per block).
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

// last request r with offsets[r] <= idx (offsets ascending, offsets[batch] > idx)
__device__ __forceinline__ int owner_of(const int64_t* __restrict__ offsets, int batch, int64_t idx) {
  int lo = 0, hi = batch - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (offsets[mid] <= idx) lo = mid; else hi = mid - 1;
  }
  return lo;
}

__global__ __launch_bounds__(256) void prefix_digest_kernel(const int32_t* __restrict__ tokens,
                                                            const int64_t* __restrict__ tok_off,
                                                            const int64_t* __restrict__ key_off, int batch,
                                                            int block_tokens, int64_t total_blocks,
                                                            uint64_t* __restrict__ keys) {
  const int lane = threadIdx.x & 63;
  const int64_t blk = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (blk >= total_blocks) return;                       // whole wave leaves together
  const int r = owner_of(key_off, batch, blk);
  const int64_t b = blk - key_off[r];
  const int64_t len = tok_off[r + 1] - tok_off[r];
  const int64_t left = len - b * block_tokens;
  const int nb = left < block_tokens ? (int)left : block_tokens;
  const int32_t* t = tokens + tok_off[r] + b * block_tokens;
  uint64_t sum = 0;
  for (int j = lane; j < nb; j += 64) sum += mix64((uint64_t)(uint32_t)t[j] + ((uint64_t)j << 32));
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const uint32_t lo = __shfl_xor((uint32_t)sum, d, 64), hi = __shfl_xor((uint32_t)(sum >> 32), d, 64);
    sum += ((uint64_t)hi << 32) | lo;
  }
  if (lane == 0) keys[blk] = mix64(sum + (uint64_t)nb);
}

__global__ __launch_bounds__(64) void prefix_chain_kernel(const int64_t* __restrict__ key_off, int batch,
                                                          uint64_t* __restrict__ keys) {
  const int r = blockIdx.x * 64 + threadIdx.x;
  if (r >= batch) return;
  uint64_t prev = 0;
  for (int64_t i = key_off[r]; i < key_off[r + 1]; ++i) {
    const uint64_t digest = keys[i];
    const uint64_t key = i == key_off[r] ? mix64(digest ^ 0x243F6A8885A308D3ull)
                                         : mix64(digest ^ (((prev << 23) | (prev >> 41)) * 0x9E3779B97F4A7C15ull));
    keys[i] = key;
    prev = key;
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
                              int block_tokens, int64_t total_blocks, uint64_t* keys, hipStream_t stream) {
  (void)hipGetLastError();
  prefix_digest_kernel<<<(unsigned)((total_blocks + 3) / 4), 256, 0, stream>>>(tokens, tok_off, key_off, batch,
                                                                               block_tokens, total_blocks, keys);
  prefix_chain_kernel<<<(unsigned)((batch + 63) / 64), 64, 0, stream>>>(key_off, batch, keys);
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
