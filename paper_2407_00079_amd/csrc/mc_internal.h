// Internal declarations shared by the C-ABI front end and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mc.h"
#include "mc_types.h"

namespace mc {

struct AttnArgs {
  const void* q;
  const void* k_pool;
  const void* v_pool;
  const int32_t* block_tables;
  void* out;
  float* lse;
  const AttnItem* items;
  const AttnReq* reqs;
  int32_t Hq, Hkv, G, max_pages;
  int32_t head_dim;   // bf16: 128 or 64; fp32: 64
  float scale_log2e;  // softmax scale * log2(e): scores go through exp2
  int32_t n_items;
  // split launches (kv_splits > 0): partial results go to o_parts [kv_splits, rows_total, D] fp32 and
  // lse_parts [kv_splits, rows_total] instead of out / lse
  int32_t kv_splits;
  int64_t rows_total;  // total_new_tokens * Hq
  float* o_parts;
  float* lse_parts;
};

// enqueue the attention kernel over args.n_items work items
hipError_t launch_attn(int dtype, const AttnArgs& args, hipStream_t stream);

// the bf16 instantiation (attn_prefill_bf16.hip), reached through launch_attn
hipError_t launch_attn_bf16(const AttnArgs& args, hipStream_t stream);

// enqueue the merge of kv_splits partial results over `rows` rows into out (dtype) and lse (or null)
hipError_t launch_attn_merge(int dtype, int head_dim, const float* o_parts, const float* lse_parts, int kv_splits, int64_t rows,
                             void* out, float* lse, hipStream_t stream);

// enqueue gather (pack) or scatter (unpack) of n pages of page_bytes for K and V; `order` (or null)
// lists the positions of page_ids in the order the workgroups should take them
hipError_t launch_kv_copy(bool pack, const void* k_src, const void* v_src, void* k_dst, void* v_dst,
                          const int32_t* page_ids, const int32_t* order, int64_t n, int64_t page_bytes,
                          hipStream_t stream);

// enqueue the computation of order[r] = position of the r-th smallest page id (stable)
hipError_t launch_kv_page_order(const int32_t* page_ids, int64_t n, int32_t* order, hipStream_t stream);

// enqueue the count of ids outside [0, num_pages) into report[0] and the first such position (n if none) into report[1]
hipError_t launch_kv_check_page_ids(const int32_t* page_ids, int64_t n, int64_t num_pages, int32_t* report,
                                    hipStream_t stream);

// enqueue the scatter of total_new tokens' K/V rows (row_bytes = 256 or 128 per KV head) into their page slots
hipError_t launch_kv_append(const void* k_new, const void* v_new, void* k_pool, void* v_pool,
                            const int32_t* block_tables, int32_t max_pages, const AttnReq* reqs, int32_t batch,
                            int64_t total_new, int32_t Hkv, int32_t row_bytes, hipStream_t stream);

// enqueue digest + chain kernels (offset tables on the device; max_blocks = most blocks of any request)
hipError_t launch_prefix_hash(const int32_t* tokens, const int64_t* tok_off, const int64_t* key_off, int batch,
                              int block_tokens, int64_t max_blocks, uint64_t* keys, hipStream_t stream);

// enqueue match + best kernels over batch requests and n_inst instances (offset tables on the device)
hipError_t launch_prefix_match(const uint64_t* keys, const int64_t* key_off, int batch, const uint64_t* cache_keys,
                               const int64_t* cache_off, int n_inst, int32_t* prefix_len, int32_t* best_len,
                               int32_t* best_inst, hipStream_t stream);

}  // namespace mc
