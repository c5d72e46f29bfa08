// Layer-wise KV page movement (paper Section 5.2: per-layer KVCache load before
// attention, store after it): gather scattered pages into a contiguous per-layer
// buffer (pack) and scatter such a buffer into scattered pages (unpack).
//
// Pure HBM traffic, no arithmetic: every byte is read once and written once with
// 128-bit nontemporal accesses.  One workgroup moves one 8 KiB slice of one page;
// its page id is a single uniform (scalar) load.  Many small workgroups (16 Ki of
// them for a 32 KiB-page layer) measured best here: slices of 4..32 KiB, 64..1024
// threads, and persistent grids all land within a few percent of each other, at
// the rate the HBM sustains for a read+write mix.
//
// Also here, all of them byte movers or integer scans over page id lists: the ranking of a page
// list by pool address (so that the scattered side of a copy can walk the pool front to back),
// the range check of an id list, and the append of a chunk's new K/V rows into their page slots.
#include "mc_internal.h"

namespace mc {
namespace {

constexpr int kThreads = 512;
constexpr int kUnroll = 1;                        // 16-byte vectors per thread
constexpr int kSliceVecs = kThreads * kUnroll;    // 8 KiB per workgroup
static_assert(kSliceVecs == kKvCopySliceVecs, "the host sizes the copy grid with kKvCopySliceVecs");

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <bool kPack>
__global__ __launch_bounds__(kThreads) void kv_copy_kernel(const u32x4* __restrict__ k_src,
                                                           const u32x4* __restrict__ v_src,
                                                           u32x4* __restrict__ k_dst,
                                                           u32x4* __restrict__ v_dst,
                                                           const int32_t* __restrict__ page_ids,
                                                           const int32_t* __restrict__ order,
                                                           int64_t page_vecs, int slices_per_page) {
  const int turn = blockIdx.x / slices_per_page;
  const int slice = blockIdx.x - turn * slices_per_page;
  // Workgroups start in blockIdx order.  With `order` (list positions by ascending pool page) the
  // scattered side of the copy walks the pool in address order, which the HBM takes better
  // than a random walk (unpack: 5.6 -> 6.1 TB/s on a 32 KiB-page layer); what is copied where is
  // the same either way.
  const int page = order != nullptr ? order[turn] : turn;
  const int64_t pool_page = page_ids[page];
  const u32x4* src = blockIdx.y ? v_src : k_src;
  u32x4* dst = blockIdx.y ? v_dst : k_dst;
  // pack: pool page -> list position; unpack: list position -> pool page
  src += (kPack ? pool_page : (int64_t)page) * page_vecs;
  dst += (kPack ? (int64_t)page : pool_page) * page_vecs;

  const int64_t first = (int64_t)slice * kSliceVecs + threadIdx.x;
  u32x4 v[kUnroll];
  if (first + (kUnroll - 1) * kThreads < page_vecs) {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(src + first + u * kThreads);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) __builtin_nontemporal_store(v[u], dst + first + u * kThreads);
  } else {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      if (first + u * kThreads < page_vecs) v[u] = __builtin_nontemporal_load(src + first + u * kThreads);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      if (first + u * kThreads < page_vecs) __builtin_nontemporal_store(v[u], dst + first + u * kThreads);
  }
}

// order[r] = the list position whose pool page is the r-th smallest (ties: lower position first),
// i.e. the rank of the 64-bit key (page id, list position).  Rank by counting, the keys staged
// through LDS in chunks and read back two per LDS instruction, one compare per key:
// O(n^2 / threads), meant to be run once per request - the list is the same for every layer.
// Slots past the end of the list hold the largest key and count nothing.
__global__ __launch_bounds__(256) void kv_page_order_kernel(const int32_t* __restrict__ page_ids, int64_t n,
                                                            int32_t* __restrict__ order) {
  typedef uint64_t u64x2 __attribute__((ext_vector_type(2)));
  __shared__ u64x2 chunk[512];
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  // ids are not negative and positions stay below 2^20: (id << 32) | position orders as the pair does
  const uint64_t mine = i < n ? ((uint64_t)(uint32_t)page_ids[i] << 32) | (uint64_t)i : 0;
  int64_t rank = 0;
  for (int64_t base = 0; base < n; base += 1024) {
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      u64x2 v;
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int64_t at = base + (threadIdx.x + h * 256) * 2 + e;
        v[e] = at < n ? ((uint64_t)(uint32_t)page_ids[at] << 32) | (uint64_t)at : ~0ull;
      }
      chunk[threadIdx.x + h * 256] = v;
    }
    __syncthreads();
    int r = 0;
#pragma unroll 8
    for (int t = 0; t < 512; ++t) {
      const u64x2 o = chunk[t];
      r += (o[0] < mine) + (o[1] < mine);
    }
    rank += r;
  }
  if (i < n) order[rank] = (int32_t)i;
}

// Range check of a page id list (debugging aid): a one-thread kernel resets the report, then every
// wave counts its out-of-range ids and adds them with one atomic; the first position by atomicMin.
__global__ void kv_check_reset_kernel(int32_t* __restrict__ report, int32_t n) {
  report[0] = 0;
  report[1] = n;
}

__global__ __launch_bounds__(256) void kv_check_page_ids_kernel(const int32_t* __restrict__ page_ids, int64_t n,
                                                                int64_t num_pages, int32_t* __restrict__ report) {
  int count = 0;
  int64_t first = n;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t id = page_ids[i];
    if (id < 0 || id >= num_pages) {
      ++count;
      first = i < first ? i : first;
    }
  }
  if (__builtin_amdgcn_ballot_w64(count != 0) == 0) return;    // the usual case: nothing to report
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    count += __shfl_xor(count, d, 64);
    const int other = __shfl_xor((int)first, d, 64);
    first = other < first ? other : first;
  }
  if ((threadIdx.x & 63) == 0) {
    atomicAdd(report, count);
    atomicMin(report + 1, (int)first);
  }
}

// Append (paper Section 3 step 2: the chunk's new KVCache is kept in the request's pages):
// one thread moves one 16-byte granule of one (token, KV head) row of K and of V.  The request
// of a token is found by bisection of the per-request table; a row has 1 << gran_shift granules
// (256 bytes for bf16 head_dim 128 and fp32 head_dim 64, 128 bytes for bf16 head_dim 64).
__global__ __launch_bounds__(256) void kv_append_kernel(const u32x4* __restrict__ k_new, const u32x4* __restrict__ v_new,
                                                        u32x4* __restrict__ k_pool, u32x4* __restrict__ v_pool,
                                                        const int32_t* __restrict__ block_tables, int32_t max_pages,
                                                        const AttnReq* __restrict__ reqs, int32_t batch,
                                                        int64_t total_vecs, int32_t Hkv, int32_t gran_shift) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total_vecs) return;
  const int gran = (int)(idx & ((1 << gran_shift) - 1));
  const int64_t row = idx >> gran_shift;        // (token, head)
  const int g = (int)(row % Hkv);
  const int32_t tok = (int32_t)(row / Hkv);
  int lo = 0, hi = batch - 1;                   // last request with q_off <= tok and at least one token
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (reqs[mid].q_off <= tok) lo = mid; else hi = mid - 1;
  }
  // requests without new tokens share their q_off with the next one: bisection lands on the
  // last of such a run, which is the one that owns the token
  const AttnReq rq = reqs[lo];
  const int32_t pos = rq.prefix + (tok - rq.q_off);
  const int64_t page = block_tables[(int64_t)lo * max_pages + (pos >> 4)];
  const int64_t dst = ((((page * Hkv + g) << 4) + (pos & 15)) << gran_shift) + gran;
  k_pool[dst] = k_new[idx];
  v_pool[dst] = v_new[idx];
}

}  // namespace

hipError_t launch_kv_page_order(const int32_t* page_ids, int64_t n, int32_t* order, hipStream_t stream) {
  (void)hipGetLastError();
  kv_page_order_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(page_ids, n, order);
  return hipGetLastError();
}

hipError_t launch_kv_check_page_ids(const int32_t* page_ids, int64_t n, int64_t num_pages, int32_t* report,
                                    hipStream_t stream) {
  (void)hipGetLastError();
  kv_check_reset_kernel<<<1, 1, 0, stream>>>(report, (int32_t)n);
  const int64_t blocks = (n + 255) / 256;
  kv_check_page_ids_kernel<<<(unsigned)(blocks < 4096 ? blocks : 4096), 256, 0, stream>>>(page_ids, n, num_pages, report);
  return hipGetLastError();
}

hipError_t launch_kv_append(const void* k_new, const void* v_new, void* k_pool, void* v_pool,
                            const int32_t* block_tables, int32_t max_pages, const AttnReq* reqs, int32_t batch,
                            int64_t total_new, int32_t Hkv, int32_t row_bytes, hipStream_t stream) {
  const int32_t gran_shift = row_bytes == 256 ? 4 : 3;      // 256- or 128-byte rows
  const int64_t total_vecs = (total_new * Hkv) << gran_shift;
  (void)hipGetLastError();
  kv_append_kernel<<<(unsigned)((total_vecs + 255) / 256), 256, 0, stream>>>(
      (const u32x4*)k_new, (const u32x4*)v_new, (u32x4*)k_pool, (u32x4*)v_pool, block_tables, max_pages, reqs, batch,
      total_vecs, Hkv, gran_shift);
  return hipGetLastError();
}

hipError_t launch_kv_copy(bool pack, const void* k_src, const void* v_src, void* k_dst, void* v_dst,
                          const int32_t* page_ids, const int32_t* order, int64_t n, int64_t page_bytes,
                          hipStream_t stream) {
  const int64_t page_vecs = page_bytes / 16;
  const int slices = (int)((page_vecs + kSliceVecs - 1) / kSliceVecs);
  dim3 grid((unsigned)(n * slices), 2, 1);
  (void)hipGetLastError();   // drop any stale error of earlier, unrelated runtime calls
  if (pack)
    kv_copy_kernel<true><<<grid, kThreads, 0, stream>>>((const u32x4*)k_src, (const u32x4*)v_src, (u32x4*)k_dst,
                                                        (u32x4*)v_dst, page_ids, order, page_vecs, slices);
  else
    kv_copy_kernel<false><<<grid, kThreads, 0, stream>>>((const u32x4*)k_src, (const u32x4*)v_src, (u32x4*)k_dst,
                                                         (u32x4*)v_dst, page_ids, order, page_vecs, slices);
  return hipGetLastError();
}

}  // namespace mc
