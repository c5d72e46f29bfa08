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
#include "mc_internal.h"

namespace mc {
namespace {

constexpr int kThreads = 512;
constexpr int kUnroll = 1;                        // 16-byte vectors per thread
constexpr int kSliceVecs = kThreads * kUnroll;    // 8 KiB per workgroup

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <bool kPack>
__global__ __launch_bounds__(kThreads) void kv_copy_kernel(const u32x4* __restrict__ k_src,
                                                           const u32x4* __restrict__ v_src,
                                                           u32x4* __restrict__ k_dst,
                                                           u32x4* __restrict__ v_dst,
                                                           const int32_t* __restrict__ page_ids,
                                                           int64_t page_vecs, int slices_per_page) {
  const int page = blockIdx.x / slices_per_page;
  const int slice = blockIdx.x - page * slices_per_page;
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

}  // namespace

int kv_copy_slice_vecs() { return kSliceVecs; }

hipError_t launch_kv_copy(bool pack, const void* k_src, const void* v_src, void* k_dst, void* v_dst,
                          const int32_t* page_ids, int64_t n, int64_t page_bytes, hipStream_t stream) {
  const int64_t page_vecs = page_bytes / 16;
  const int slices = (int)((page_vecs + kSliceVecs - 1) / kSliceVecs);
  dim3 grid((unsigned)(n * slices), 2, 1);
  (void)hipGetLastError();   // drop any stale error of earlier, unrelated runtime calls
  if (pack)
    kv_copy_kernel<true><<<grid, kThreads, 0, stream>>>((const u32x4*)k_src, (const u32x4*)v_src, (u32x4*)k_dst,
                                                        (u32x4*)v_dst, page_ids, page_vecs, slices);
  else
    kv_copy_kernel<false><<<grid, kThreads, 0, stream>>>((const u32x4*)k_src, (const u32x4*)v_src, (u32x4*)k_dst,
                                                         (u32x4*)v_dst, page_ids, page_vecs, slices);
  return hipGetLastError();
}

}  // namespace mc
