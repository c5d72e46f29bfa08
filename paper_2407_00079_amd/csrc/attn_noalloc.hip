// mc_prefill_attn_paged_noalloc: the whole-row attention call for callers that cannot allocate
// (code under HIP graph capture, serving loops and harnesses that forbid hipMalloc).
//
// mc_prefill_attn_paged keeps its work list and request table in a caller-supplied workspace and
// uploads them from pinned host memory.  Here both live in a file-scope device array, and the
// list is BUILT ON THE DEVICE by a small kernel that gets the batch's lengths as a kernel
// argument: no workspace, no upload, no allocation of any kind (no hipMalloc, hipHostMalloc or
// hipFree; no host heap either).  The attention kernel is the one every other entry point runs.
//
// The list the kernel writes is the list mc::host::build_work_list makes, item for item: the
// items of each of the 8 per-XCD lists in order of falling key count (ties in enumeration order),
// dealt round-robin.  Key counts rise with the tile index inside a (request, KV head), so the
// rank of an item inside its list is a sum of bisection results over the requests - no sort.
#include <mutex>

#include "host_plan.h"
#include "mc_internal.h"

namespace mc {
namespace {

constexpr int kMaxBatch = MC_NOALLOC_MAX_BATCH;
constexpr int kMaxItems = MC_NOALLOC_MAX_ITEMS;
constexpr size_t kReqsOffset = sizeof(AttnItem) * (size_t)kMaxItems;
constexpr size_t kScratchBytes = kReqsOffset + sizeof(AttnReq) * (size_t)kMaxBatch;

// Work list, then request table.  One copy per GPU the library runs on, held until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress: the address kernels and
// runtime calls take is the one that call returns (scratch_of_current_device below).
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

struct BatchLens {           // 1 KiB, passed to the kernel by value
  int32_t prefix[kMaxBatch];
  int32_t chunk[kMaxBatch];
};

__device__ __forceinline__ int64_t tile_cost(int32_t P, int32_t C, int G, int t) {
  // keys the last row of tile t sees (host_plan.cpp: build_work_list)
  const int64_t tok_last = ((int64_t)t * kAttnTileRows + kAttnTileRows - 1) / G;
  return (int64_t)P + (tok_last < C - 1 ? tok_last : C - 1) + 1;
}

// first tile of the request whose cost is >= c (strict == false) or > c (strict == true); tiles if none
__device__ __forceinline__ int first_tile_at_least(int32_t P, int32_t C, int G, int tiles, int64_t c, bool strict) {
  int lo = 0, hi = tiles;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    const int64_t v = tile_cost(P, C, G, mid);
    if (strict ? v > c : v >= c) hi = mid;
    else lo = mid + 1;
  }
  return lo;
}

// KV heads g in [0, upto) with (r * Hkv + g) % 8 == x
__device__ __forceinline__ int heads_in_list(int r, int Hkv, int x, int upto) {
  const int t = (x - r * Hkv) & (kXcds - 1);       // smallest such g
  return upto > t ? (upto - t - 1) / kXcds + 1 : 0;
}

__global__ __launch_bounds__(256) void build_list_kernel(const BatchLens lens, int batch, int Hkv, int G, int page_size,
                                                         AttnItem* __restrict__ items, AttnReq* __restrict__ reqs,
                                                         int n_items) {
  __shared__ int s_tiles[kMaxBatch];        // tiles of stacked rows per (request, KV head)
  __shared__ int s_first[kMaxBatch + 1];    // index of the request's first item in enumeration order
  __shared__ int s_qoff[kMaxBatch];
  __shared__ int s_size[kXcds];             // items per list
  const int tid = threadIdx.x;
  if (tid < batch) s_tiles[tid] = (int)(((int64_t)lens.chunk[tid] * G + kAttnTileRows - 1) / kAttnTileRows);
  __syncthreads();
  if (tid == 0) {
    int first = 0, q = 0;
    for (int r = 0; r < batch; ++r) {
      s_first[r] = first;
      s_qoff[r] = q;
      first += Hkv * s_tiles[r];
      q += lens.chunk[r];
    }
    s_first[batch] = first;
  }
  if (tid >= 64 && tid < 64 + kXcds) {      // another wave than thread 0's
    const int x = tid - 64;
    int size = 0;
    for (int r = 0; r < batch; ++r) size += heads_in_list(r, Hkv, x, Hkv) * s_tiles[r];
    s_size[x] = size;
  }
  __syncthreads();

  const int e = blockIdx.x * 256 + tid;
  if (e < batch)
    reqs[e] = AttnReq{s_qoff[e], lens.prefix[e], lens.chunk[e],
                      (int32_t)(((int64_t)lens.prefix[e] + lens.chunk[e] + page_size - 1) / page_size)};
  if (e >= n_items) return;

  // which (request, KV head, tile) is item e of the enumeration
  int lo = 0, hi = batch - 1;               // last request with s_first <= e and at least one tile
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (s_first[mid] <= e) lo = mid;
    else hi = mid - 1;
  }
  const int r = lo;                         // requests without tiles share s_first with the next one: lo is past them
  const int rem = e - s_first[r];
  const int g = rem / s_tiles[r], t = rem - g * s_tiles[r];
  const int x = (r * Hkv + g) & (kXcds - 1);
  const int64_t c = tile_cost(lens.prefix[r], lens.chunk[r], G, t);

  // rank inside list x: items with more keys, and items with as many that were enumerated earlier
  int rank = 0;
  for (int o = 0; o < batch; ++o) {
    const int tiles = s_tiles[o];
    const int heads = heads_in_list(o, Hkv, x, Hkv);
    if (tiles == 0 || heads == 0) continue;
    const int ge = tiles - first_tile_at_least(lens.prefix[o], lens.chunk[o], G, tiles, c, false);   // cost >= c
    const int gt = tiles - first_tile_at_least(lens.prefix[o], lens.chunk[o], G, tiles, c, true);    // cost >  c
    if (o < r) rank += heads * ge;
    else if (o > r) rank += heads * gt;
    else {
      const int before = heads_in_list(o, Hkv, x, g);         // heads of this request enumerated before g
      // own (request, head): later tiles have more keys; of the tiles with as many, those before t
      rank += before * ge + (heads - before - 1) * gt + gt + (t - (tiles - ge));
    }
  }
  // round-robin deal of the 8 lists, exhausted lists skipped: round `rank` comes after min(size, rank)
  // items of every list, and after the items of this round from the lists before x
  int pos = 0;
#pragma unroll
  for (int y = 0; y < kXcds; ++y) {
    const int size = s_size[y];
    pos += (size < rank ? size : rank) + (y < x && size > rank ? 1 : 0);
  }
  items[pos] = AttnItem{r, g, t * kAttnTileRows, 0};
}

// Device address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices] = {};

void* scratch_of_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace
}  // namespace mc

extern "C" mc_status mc_prefill_attn_paged_noalloc(const mc_attn_params* p, const void* q, const void* k_pool,
                                                   const void* v_pool, const int32_t* block_tables,
                                                   int32_t max_pages_per_req, const int32_t* prefix_lens,
                                                   const int32_t* new_lens, int32_t batch, void* out, float* lse,
                                                   void* hip_stream) {
  using namespace mc;
  using namespace mc::host;
  mc_status st = check_params(p);
  if (st != MC_OK) return st;
  if (batch < 0 || max_pages_per_req < 0) return MC_ERR_SHAPE;
  if (batch == 0) return MC_OK;
  if (prefix_lens == nullptr || new_lens == nullptr) return MC_ERR_NULL;
  int64_t total_new = 0;
  int32_t need_pages = 0;
  st = check_lens(p, prefix_lens, new_lens, batch, &total_new, &need_pages);
  if (st != MC_OK) return st;
  if (total_new == 0) return MC_OK;
  st = check_attn_buffers(false, q, k_pool, v_pool, block_tables, batch, max_pages_per_req, need_pages, out, lse,
                          nullptr, nullptr, nullptr);
  if (st != MC_OK) return st;
  st = check_list_range(p, batch, total_new, 0);
  if (st != MC_OK) return st;
  const int64_t n_items = count_items(p, new_lens, batch);
  if (batch > kMaxBatch || n_items > kMaxItems) return MC_ERR_RANGE;   // beyond the fixed scratch array

  char* base = reinterpret_cast<char*>(scratch_of_current_device());
  if (base == nullptr) return MC_ERR_HIP;
  AttnItem* items = reinterpret_cast<AttnItem*>(base);
  AttnReq* reqs = reinterpret_cast<AttnReq*>(base + kReqsOffset);

  BatchLens lens;
  for (int32_t r = 0; r < batch; ++r) {
    lens.prefix[r] = prefix_lens[r];
    lens.chunk[r] = new_lens[r];
  }
  for (int32_t r = batch; r < kMaxBatch; ++r) lens.prefix[r] = lens.chunk[r] = 0;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const int G = p->num_q_heads / p->num_kv_heads;
  (void)hipGetLastError();
  build_list_kernel<<<(unsigned)((n_items + 255) / 256), 256, 0, stream>>>(lens, batch, p->num_kv_heads, G,
                                                                            p->page_size, items, reqs, (int)n_items);
  if (hipGetLastError() != hipSuccess) return MC_ERR_HIP;

  AttnArgs args;
  args.q = q;
  args.k_pool = k_pool;
  args.v_pool = v_pool;
  args.block_tables = block_tables;
  args.out = out;
  args.lse = lse;
  args.items = items;
  args.reqs = reqs;
  args.Hq = p->num_q_heads;
  args.Hkv = p->num_kv_heads;
  args.G = G;
  args.max_pages = max_pages_per_req;
  args.head_dim = p->head_dim;
  args.scale_log2e = attn_scale_log2e(p);
  args.n_items = (int32_t)n_items;
  args.kv_splits = 0;
  args.rows_total = total_new * p->num_q_heads;
  args.o_parts = nullptr;
  args.lse_parts = nullptr;
  if (launch_attn(p->dtype, args, stream) != hipSuccess) return MC_ERR_HIP;
  return MC_OK;
}
