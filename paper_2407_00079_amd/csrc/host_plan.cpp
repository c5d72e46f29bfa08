// Host-side planning and validation (no HIP calls; see host_plan.h).
#include "host_plan.h"

#include <algorithm>
#include <cmath>
#include <cstring>

namespace mc {
namespace host {

mc_status check_params(const mc_attn_params* p) {
  if (p == nullptr) return MC_ERR_NULL;
  if (p->num_q_heads <= 0 || p->num_kv_heads <= 0 || p->head_dim <= 0 || p->page_size <= 0 || p->num_pages <= 0)
    return MC_ERR_SHAPE;
  if (p->num_q_heads % p->num_kv_heads != 0) return MC_ERR_SHAPE;
  if (p->dtype != MC_DTYPE_BF16 && p->dtype != MC_DTYPE_F32) return MC_ERR_UNSUPPORTED;
  if (p->page_size != 16) return MC_ERR_UNSUPPORTED;
  if (p->dtype == MC_DTYPE_BF16 && p->head_dim != 128 && p->head_dim != 64) return MC_ERR_UNSUPPORTED;
  if (p->dtype == MC_DTYPE_F32 && p->head_dim != 64) return MC_ERR_UNSUPPORTED;
  if (!(p->softmax_scale >= 0.f) || std::isinf(p->softmax_scale)) return MC_ERR_SHAPE;
  return MC_OK;
}

float attn_scale_log2e(const mc_attn_params* p) {
  const double scale = p->softmax_scale > 0.f ? (double)p->softmax_scale : 1.0 / std::sqrt((double)p->head_dim);
  return (float)(scale * 1.4426950408889634);
}

size_t max_items(const mc_attn_params* p, int32_t batch, int64_t total_new_tokens, int32_t kv_splits) {
  const int64_t G = p->num_q_heads / p->num_kv_heads;
  return (size_t)(p->num_kv_heads * ((total_new_tokens * G) / kAttnTileRows + batch)) * (size_t)kv_splits;
}

size_t list_bytes(const mc_attn_params* p, int32_t batch, int64_t total_new_tokens, int32_t kv_splits) {
  return sizeof(AttnItem) * max_items(p, batch, total_new_tokens, kv_splits) + sizeof(AttnReq) * (size_t)batch + 64;
}

mc_status check_lens(const mc_attn_params* p, const int32_t* prefix_lens, const int32_t* new_lens, int32_t batch,
                     int64_t* total_new, int32_t* need_pages) {
  *total_new = 0;
  *need_pages = 0;
  for (int32_t r = 0; r < batch; ++r) {
    if (prefix_lens[r] < 0 || new_lens[r] < 0) return MC_ERR_SHAPE;
    const int64_t len = (int64_t)prefix_lens[r] + new_lens[r];
    if (len > INT32_MAX - 1024) return MC_ERR_RANGE;
    if (new_lens[r] > 0) {
      const int32_t pages = (int32_t)((len + p->page_size - 1) / p->page_size);
      *need_pages = pages > *need_pages ? pages : *need_pages;
    }
    *total_new += new_lens[r];
  }
  return MC_OK;
}

mc_status check_attn_buffers(bool split, const void* q, const void* k_pool, const void* v_pool,
                             const int32_t* block_tables, int32_t batch, int32_t max_pages_per_req, int32_t need_pages,
                             const void* out, const float* lse, const float* o_parts, const float* lse_parts,
                             const void* workspace) {
  if (max_pages_per_req < need_pages) return MC_ERR_SHAPE;
  if (q == nullptr || k_pool == nullptr || v_pool == nullptr || block_tables == nullptr) return MC_ERR_NULL;
  if (split ? (o_parts == nullptr || lse_parts == nullptr) : out == nullptr) return MC_ERR_NULL;
  if (!aligned16(q) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(out) || !aligned16(workspace) ||
      !aligned16(o_parts) || !aligned4(block_tables) || !aligned4(lse) || !aligned4(lse_parts))
    return MC_ERR_ALIGN;
  if ((int64_t)batch * max_pages_per_req > INT32_MAX) return MC_ERR_RANGE;
  return MC_OK;
}

mc_status check_list_range(const mc_attn_params* p, int32_t batch, int64_t total_new, int32_t kv_splits) {
  if (total_new * p->num_q_heads > INT32_MAX) return MC_ERR_RANGE;
  if (max_items(p, batch, total_new, kv_splits > 0 ? kv_splits : 1) > (size_t)INT32_MAX) return MC_ERR_RANGE;
  return MC_OK;
}

void build_work_list(const mc_attn_params* p, const int32_t* prefix_lens, const int32_t* new_lens, int32_t batch,
                     int32_t kv_splits, std::vector<AttnReq>& reqs, std::vector<AttnItem>& items) {
  const bool split = kv_splits > 0;
  const int G = p->num_q_heads / p->num_kv_heads;
  const int rows = kAttnTileRows;
  reqs.assign((size_t)batch, AttnReq{});
  struct Keyed {
    int64_t cost;
    AttnItem it;
  };
  std::vector<Keyed> lanes[kXcds];
  int64_t q_off = 0;
  for (int32_t r = 0; r < batch; ++r) {
    const int32_t P = prefix_lens[r], C = new_lens[r];
    reqs[(size_t)r] = {(int32_t)q_off, P, C, (int32_t)(((int64_t)P + C + p->page_size - 1) / p->page_size)};
    q_off += C;
    const int64_t n_rows = (int64_t)C * G;
    for (int32_t g = 0; g < p->num_kv_heads; ++g)
      for (int64_t row0 = 0; row0 < n_rows; row0 += rows) {
        const int64_t tok_last = std::min<int64_t>(C - 1, (row0 + rows - 1) / G);
        const int64_t keys = P + tok_last + 1;                 // keys the tile's last row sees
        if (!split) {
          lanes[(r * p->num_kv_heads + g) % kXcds].push_back({keys, {r, g, (int32_t)row0, 0}});
          continue;
        }
        // slices of whole 64-key tiles, ceil(tiles of the request / kv_splits) each; every slice gets
        // an item, also one past what the tile can see (it writes zeros and -inf)
        const int64_t per =
            ((((int64_t)P + C + kAttnTileKeys - 1) / kAttnTileKeys) + kv_splits - 1) / kv_splits * kAttnTileKeys;
        for (int32_t sl = 0; sl < kv_splits; ++sl) {
          const int64_t cost = std::max<int64_t>(0, std::min<int64_t>(keys, (sl + 1) * per) - sl * per);
          lanes[(r * p->num_kv_heads + g + sl) % kXcds].push_back({cost, {r, g, (int32_t)row0, sl}});
        }
      }
  }
  size_t n_items = 0;
  for (auto& l : lanes) {
    std::stable_sort(l.begin(), l.end(), [](const Keyed& a, const Keyed& b) { return a.cost > b.cost; });
    n_items += l.size();
  }
  items.clear();
  items.reserve(n_items);
  size_t cur[kXcds] = {0};
  int x = 0;
  while (items.size() < n_items) {
    // next non-empty lane, starting from the one whose turn it is
    int tries = 0;
    while (cur[x] >= lanes[x].size() && tries < kXcds) {
      x = (x + 1) % kXcds;
      ++tries;
    }
    items.push_back(lanes[x][cur[x]++].it);
    x = (x + 1) % kXcds;
  }
}

int64_t count_items(const mc_attn_params* p, const int32_t* new_lens, int32_t batch) {
  const int64_t G = p->num_q_heads / p->num_kv_heads;
  int64_t n = 0;
  for (int32_t r = 0; r < batch; ++r)
    n += (int64_t)p->num_kv_heads * (((int64_t)new_lens[r] * G + kAttnTileRows - 1) / kAttnTileRows);
  return n;
}

mc_status check_plan(const mc_attn_params* p, const mc_attn_plan* plan, bool want_split) {
  if (plan == nullptr) return MC_ERR_NULL;
  if (plan->num_q_heads != p->num_q_heads || plan->num_kv_heads != p->num_kv_heads || plan->dtype != (int32_t)p->dtype ||
      plan->n_items < 0 || plan->batch < 0 || plan->total_new_tokens < 0 || plan->reqs_offset < 0 ||
      (plan->reqs_offset & 15) != 0 || plan->kv_splits < 0 || plan->kv_splits > MC_MAX_KV_SPLITS)
    return MC_ERR_SHAPE;
  if (want_split != (plan->kv_splits > 0)) return MC_ERR_SHAPE;
  return MC_OK;
}

mc_status plan_items(const mc_attn_params* p, const int32_t* prefix_lens, const int32_t* new_lens, int32_t batch,
                     int32_t kv_splits, int32_t* items, int64_t capacity, int64_t* n_items) {
  mc_status st = check_params(p);
  if (st != MC_OK) return st;
  if (batch < 0 || kv_splits < 0 || kv_splits > MC_MAX_KV_SPLITS || capacity < 0) return MC_ERR_SHAPE;
  if (n_items == nullptr || (batch > 0 && (prefix_lens == nullptr || new_lens == nullptr))) return MC_ERR_NULL;
  if (capacity > 0 && items == nullptr) return MC_ERR_NULL;
  int64_t total_new = 0;
  int32_t need_pages = 0;
  st = check_lens(p, prefix_lens, new_lens, batch, &total_new, &need_pages);
  if (st != MC_OK) return st;
  st = check_list_range(p, batch, total_new, kv_splits);
  if (st != MC_OK) return st;
  std::vector<AttnReq> reqs;
  std::vector<AttnItem> list;
  build_work_list(p, prefix_lens, new_lens, batch, kv_splits, reqs, list);
  *n_items = (int64_t)list.size();
  if ((int64_t)list.size() > capacity) return capacity == 0 && items == nullptr ? MC_OK : MC_ERR_WORKSPACE;
  static_assert(sizeof(AttnItem) == 4 * sizeof(int32_t), "an item is four int32");
  if (!list.empty()) std::memcpy(items, list.data(), sizeof(AttnItem) * list.size());
  return MC_OK;
}

int32_t suggest_kv_splits(const mc_attn_params* p, const int32_t* prefix_lens, const int32_t* new_lens,
                          int32_t batch) {
  if (check_params(p) != MC_OK || batch < 0) return 0;
  if (batch > 0 && (prefix_lens == nullptr || new_lens == nullptr)) return 0;
  constexpr int64_t kComputeUnits = 256;   // MI355X
  constexpr int64_t kMinTilesPerSlice = 8;
  const int64_t G = p->num_q_heads / p->num_kv_heads;
  int64_t items = 0, most_tiles = 0;
  for (int32_t r = 0; r < batch; ++r) {
    if (prefix_lens[r] < 0 || new_lens[r] < 0) return 0;
    if (new_lens[r] == 0) continue;
    items += (int64_t)p->num_kv_heads * (((int64_t)new_lens[r] * G + kAttnTileRows - 1) / kAttnTileRows);
    const int64_t tiles = ((int64_t)prefix_lens[r] + new_lens[r] + kAttnTileKeys - 1) / kAttnTileKeys;
    most_tiles = tiles > most_tiles ? tiles : most_tiles;
  }
  // Work items of about equal length run in rounds of one per compute unit: s slices turn `items`
  // items into items * s of 1/s the length, ceil(items * s / 256) / s rounds of the original
  // length, and each extra slice costs about 1 % in partial results written and merged
  // (measured at 128k context).  The cheapest count wins, the smaller one on a tie.  From four
  // full rounds on, the launch order (longest items first) already balances the tail.
  if (items == 0 || items >= 4 * kComputeUnits) return 1;
  int64_t most = most_tiles / kMinTilesPerSlice;
  most = most < MC_MAX_KV_SPLITS ? most : MC_MAX_KV_SPLITS;
  int32_t best = 1;
  double best_cost = 0.0;
  for (int64_t sl = 1; sl <= most || sl == 1; ++sl) {
    const double rounds = (double)((items * sl + kComputeUnits - 1) / kComputeUnits) / (double)sl;
    const double cost = rounds * (1.0 + 0.01 * (double)(sl - 1));
    if (sl == 1 || cost < best_cost) {
      best = (int32_t)sl;
      best_cost = cost;
    }
  }
  return best;
}

bool auto_layout(const mc_attn_params* p, const int32_t* prefix_lens, const int32_t* new_lens, int32_t batch,
                 AutoLayout* lay) {
  const int32_t s = suggest_kv_splits(p, prefix_lens, new_lens, batch);
  if (s <= 0) return false;
  int64_t total_new = 0;
  for (int32_t r = 0; r < batch; ++r) total_new += new_lens[r];
  lay->kv_splits = s;
  if (s == 1) {
    lay->list_bytes = list_bytes(p, batch, total_new);
    lay->o_off = lay->lse_off = lay->total = lay->list_bytes;
    return true;
  }
  const size_t rows = (size_t)total_new * (size_t)p->num_q_heads;
  lay->list_bytes = list_bytes(p, batch, total_new, s);
  lay->o_off = (lay->list_bytes + 255) & ~(size_t)255;
  lay->lse_off = (lay->o_off + (size_t)s * rows * (size_t)p->head_dim * sizeof(float) + 255) & ~(size_t)255;
  lay->total = lay->lse_off + (size_t)s * rows * sizeof(float);
  return true;
}

mc_status check_copy(const void* a, const void* b, int64_t num_pages, int64_t page_bytes, const int32_t* ids,
                     int64_t n, const void* c, const void* d) {
  if (num_pages < 0 || page_bytes < 0 || n < 0) return MC_ERR_SHAPE;
  if (page_bytes % 16 != 0) return MC_ERR_ALIGN;
  if (n == 0 || page_bytes == 0) return MC_OK;
  if (a == nullptr || b == nullptr || c == nullptr || d == nullptr || ids == nullptr) return MC_ERR_NULL;
  if (num_pages == 0) return MC_ERR_SHAPE;
  if (!aligned16(a) || !aligned16(b) || !aligned16(c) || !aligned16(d) || !aligned4(ids)) return MC_ERR_ALIGN;
  const int64_t slices = (page_bytes / 16 + kKvCopySliceVecs - 1) / kKvCopySliceVecs;
  if (n > INT32_MAX || n * slices > INT32_MAX) return MC_ERR_RANGE;
  return MC_OK;
}

}  // namespace host
}  // namespace mc
