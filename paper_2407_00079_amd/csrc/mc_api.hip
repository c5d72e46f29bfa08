// C-ABI front end: host-side validation, work-list construction, launches.
// Every check runs before the first HIP call, so a rejected call leaves no trace.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "host_plan.h"
#include "mc_internal.h"

namespace {

using namespace mc::host;

// bytes of one K or V row of one KV head
int32_t row_bytes_of(const mc_attn_params* p) { return p->head_dim * (p->dtype == MC_DTYPE_BF16 ? 2 : 4); }

// Pinned host slots the work list is written to before its asynchronous upload.  A slot is
// reused only after the event recorded behind its last upload has completed, so the host copy
// outlives the transfer.  A call never waits for the stream's earlier work: if every slot is
// still in flight a new one is added (up to SlotRing::kMaxSlots; only then does a call block on
// the oldest).  Which slot a call gets is decided by mc::host::SlotRing under this class's lock:
// from acquire() until in_flight() or abandon() the slot is HELD and no other thread can be
// given it.  Host memory only, 64 KiB or the largest work list seen per slot, kept until the
// process ends.
class StagingRing {
 public:
  // returns a held slot with at least `bytes` of pinned memory, or nullptr if HIP refuses
  void* acquire(size_t bytes, int* slot_out) {
    std::lock_guard<std::mutex> lock(mu_);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return nullptr;
    const SlotRing::Pick pick = ring_.pick(dev, [&](int i) { return hipEventQuery(mem_[i].ev) == hipSuccess; });
    if (pick.slot < 0) return nullptr;
    Mem& m = mem_[pick.slot];
    if (pick.is_new) {
      m = Mem{};
      if (hipEventCreateWithFlags(&m.ev, hipEventDisableTiming) != hipSuccess) {
        ring_.drop_new(pick.slot);
        return nullptr;
      }
    }
    if (pick.must_wait && hipEventSynchronize(m.ev) != hipSuccess) {
      ring_.in_flight(pick.slot);   // still not known to be done: leave it as it was
      return nullptr;
    }
    if (m.cap < bytes) {
      if (m.host != nullptr) (void)hipHostFree(m.host);
      m.host = nullptr;
      m.cap = 0;
      const size_t want = std::max<size_t>(bytes, 1 << 16);
      if (hipHostMalloc(&m.host, want, hipHostMallocDefault) != hipSuccess) {
        m.host = nullptr;
        ring_.abandon(pick.slot);
        return nullptr;
      }
      m.cap = want;
    }
    *slot_out = pick.slot;
    return m.host;
  }
  // the upload from the slot has been enqueued on `stream`: the slot is free again once the
  // stream has passed this point.  If the event cannot be recorded the stream is waited for
  // instead, so the slot never returns to the ring while a copy may still read it.
  bool release_after(int slot, hipStream_t stream) {
    std::lock_guard<std::mutex> lock(mu_);
    if (hipEventRecord(mem_[slot].ev, stream) == hipSuccess) {
      ring_.in_flight(slot);
      return true;
    }
    (void)hipStreamSynchronize(stream);
    ring_.abandon(slot);
    return false;
  }
  // nothing was enqueued from the slot
  void abandon(int slot) {
    std::lock_guard<std::mutex> lock(mu_);
    ring_.abandon(slot);
  }

 private:
  struct Mem {
    void* host = nullptr;
    size_t cap = 0;
    hipEvent_t ev = nullptr;
  };
  std::mutex mu_;
  SlotRing ring_;
  Mem mem_[SlotRing::kMaxSlots];
};

StagingRing g_staging;

}  // namespace

extern "C" {

const char* mc_status_string(mc_status s) {
  switch (s) {
    case MC_OK: return "ok";
    case MC_ERR_NULL: return "null pointer";
    case MC_ERR_SHAPE: return "bad shape";
    case MC_ERR_UNSUPPORTED: return "unsupported head_dim / page_size / dtype";
    case MC_ERR_ALIGN: return "misaligned pointer or page size";
    case MC_ERR_RANGE: return "size out of range";
    case MC_ERR_WORKSPACE: return "workspace missing or too small";
    case MC_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

size_t mc_prefill_attn_workspace_bytes(const mc_attn_params* p, int32_t batch, int64_t total_new_tokens) {
  if (check_params(p) != MC_OK || batch < 0 || total_new_tokens < 0) return 0;
  return list_bytes(p, batch, total_new_tokens);
}

}  // extern "C"

namespace {

// Build the work list and the request table of a batch and enqueue their upload into the
// workspace; fill `plan` with what a later launch needs to know on the host.  The lengths have
// passed check_lens and total_new > 0.
mc_status prepare_attn(const mc_attn_params* p, const int32_t* prefix_lens, const int32_t* new_lens, int32_t batch,
                       int32_t kv_splits, int64_t total_new, int32_t need_pages, void* workspace,
                       size_t workspace_bytes, hipStream_t stream, mc_attn_plan* plan) {
  const bool split = kv_splits > 0;
  const mc_status range = check_list_range(p, batch, total_new, kv_splits);
  if (range != MC_OK) return range;
  if (workspace == nullptr || workspace_bytes < list_bytes(p, batch, total_new, split ? kv_splits : 1))
    return MC_ERR_WORKSPACE;
  if (!aligned16(workspace)) return MC_ERR_ALIGN;

  std::vector<mc::AttnReq> reqs;
  std::vector<mc::AttnItem> items;
  build_work_list(p, prefix_lens, new_lens, batch, split ? kv_splits : 0, reqs, items);
  const size_t n_items = items.size();

  // one pinned, asynchronous copy of work list + request table
  const size_t items_bytes = sizeof(mc::AttnItem) * n_items;
  const size_t reqs_off = (items_bytes + 15) & ~(size_t)15;
  const size_t up_bytes = reqs_off + sizeof(mc::AttnReq) * reqs.size();
  int slot = -1;
  char* host = reinterpret_cast<char*>(g_staging.acquire(up_bytes, &slot));
  if (host == nullptr) return MC_ERR_HIP;
  std::memcpy(host, items.data(), items_bytes);
  std::memcpy(host + reqs_off, reqs.data(), sizeof(mc::AttnReq) * reqs.size());
  if (hipMemcpyAsync(workspace, host, up_bytes, hipMemcpyHostToDevice, stream) != hipSuccess) {
    g_staging.abandon(slot);
    return MC_ERR_HIP;
  }
  if (!g_staging.release_after(slot, stream)) return MC_ERR_HIP;

  plan->n_items = (int32_t)n_items;
  plan->batch = batch;
  plan->kv_splits = split ? kv_splits : 0;
  plan->need_pages = need_pages;
  plan->total_new_tokens = total_new;
  plan->reqs_offset = (int64_t)reqs_off;
  plan->num_q_heads = p->num_q_heads;
  plan->num_kv_heads = p->num_kv_heads;
  plan->dtype = (int32_t)p->dtype;
  plan->reserved = 0;
  return MC_OK;
}

mc_status launch_planned_attn(const mc_attn_params* p, const mc_attn_plan* plan, const void* q, const void* k_pool,
                              const void* v_pool, const int32_t* block_tables, int32_t max_pages_per_req, void* out,
                              float* lse, float* o_parts, float* lse_parts, const void* workspace,
                              hipStream_t stream) {
  const char* ws = reinterpret_cast<const char*>(workspace);
  mc::AttnArgs args;
  args.q = q;
  args.k_pool = k_pool;
  args.v_pool = v_pool;
  args.block_tables = block_tables;
  args.out = out;
  args.lse = lse;
  args.items = reinterpret_cast<const mc::AttnItem*>(ws);
  args.reqs = reinterpret_cast<const mc::AttnReq*>(ws + plan->reqs_offset);
  args.Hq = p->num_q_heads;
  args.Hkv = p->num_kv_heads;
  args.G = p->num_q_heads / p->num_kv_heads;
  args.max_pages = max_pages_per_req;
  args.head_dim = p->head_dim;
  args.scale_log2e = attn_scale_log2e(p);
  args.n_items = plan->n_items;
  args.kv_splits = plan->kv_splits;
  args.rows_total = plan->total_new_tokens * p->num_q_heads;
  args.o_parts = o_parts;
  args.lse_parts = lse_parts;
  if (mc::launch_attn(p->dtype, args, stream) != hipSuccess) return MC_ERR_HIP;
  return MC_OK;
}

// One-shot form: every check first (a rejected call enqueues nothing), then upload and launch.
mc_status attn_enqueue(const mc_attn_params* p, const void* q, const void* k_pool, const void* v_pool,
                       const int32_t* block_tables, int32_t max_pages_per_req, const int32_t* prefix_lens,
                       const int32_t* new_lens, int32_t batch, void* out, float* lse, int32_t kv_splits,
                       float* o_parts, float* lse_parts, void* workspace, size_t workspace_bytes,
                       void* hip_stream) {
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
  st = check_attn_buffers(kv_splits > 0, q, k_pool, v_pool, block_tables, batch, max_pages_per_req, need_pages, out,
                          lse, o_parts, lse_parts, workspace);
  if (st != MC_OK) return st;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  mc_attn_plan plan;
  st = prepare_attn(p, prefix_lens, new_lens, batch, kv_splits, total_new, need_pages, workspace, workspace_bytes,
                    stream, &plan);
  if (st != MC_OK) return st;
  return launch_planned_attn(p, &plan, q, k_pool, v_pool, block_tables, max_pages_per_req, out, lse, o_parts,
                             lse_parts, workspace, stream);
}

}  // namespace

extern "C" {

mc_status mc_prefill_attn_paged(const mc_attn_params* p, const void* q, const void* k_pool, const void* v_pool,
                                const int32_t* block_tables, int32_t max_pages_per_req,
                                const int32_t* prefix_lens, const int32_t* new_lens, int32_t batch, void* out,
                                float* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
  // A launch that would leave compute units idle (a small chunk behind a long prefix, or a work-item count just
  // above a multiple of the compute units) runs over key slices + merge when the caller's workspace has room
  // for the partial results; with the minimal workspace it runs whole-row.
  AutoLayout lay;
  if (workspace != nullptr && batch > 0 && prefix_lens != nullptr && new_lens != nullptr &&
      auto_layout(p, prefix_lens, new_lens, batch, &lay) && lay.kv_splits > 1 && workspace_bytes >= lay.total)
    return mc_prefill_attn_auto(p, q, k_pool, v_pool, block_tables, max_pages_per_req, prefix_lens, new_lens, batch,
                                out, lse, workspace, workspace_bytes, hip_stream);
  return attn_enqueue(p, q, k_pool, v_pool, block_tables, max_pages_per_req, prefix_lens, new_lens, batch, out, lse,
                      0, nullptr, nullptr, workspace, workspace_bytes, hip_stream);
}

size_t mc_prefill_attn_split_workspace_bytes(const mc_attn_params* p, int32_t batch, int64_t total_new_tokens,
                                             int32_t kv_splits) {
  if (check_params(p) != MC_OK || batch < 0 || total_new_tokens < 0 || kv_splits < 1 || kv_splits > MC_MAX_KV_SPLITS)
    return 0;
  return list_bytes(p, batch, total_new_tokens, kv_splits);
}

mc_status mc_prefill_attn_paged_split(const mc_attn_params* p, const void* q, const void* k_pool,
                                      const void* v_pool, const int32_t* block_tables, int32_t max_pages_per_req,
                                      const int32_t* prefix_lens, const int32_t* new_lens, int32_t batch,
                                      int32_t kv_splits, float* o_parts, float* lse_parts, void* workspace,
                                      size_t workspace_bytes, void* hip_stream) {
  if (kv_splits < 1 || kv_splits > MC_MAX_KV_SPLITS) return MC_ERR_SHAPE;
  return attn_enqueue(p, q, k_pool, v_pool, block_tables, max_pages_per_req, prefix_lens, new_lens, batch, nullptr,
                      nullptr, kv_splits, o_parts, lse_parts, workspace, workspace_bytes, hip_stream);
}

size_t mc_prefill_attn_auto_workspace_bytes(const mc_attn_params* p, const int32_t* prefix_lens,
                                            const int32_t* new_lens, int32_t batch) {
  AutoLayout lay;
  return auto_layout(p, prefix_lens, new_lens, batch, &lay) ? lay.total : 0;
}

mc_status mc_prefill_attn_auto(const mc_attn_params* p, const void* q, const void* k_pool, const void* v_pool,
                               const int32_t* block_tables, int32_t max_pages_per_req,
                               const int32_t* prefix_lens, const int32_t* new_lens, int32_t batch, void* out,
                               float* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
  AutoLayout lay;
  if (!auto_layout(p, prefix_lens, new_lens, batch, &lay) || lay.kv_splits == 1)
    // one slice, or arguments the whole-row call will name the fault of
    return attn_enqueue(p, q, k_pool, v_pool, block_tables, max_pages_per_req, prefix_lens, new_lens, batch, out, lse,
                        0, nullptr, nullptr, workspace, workspace_bytes, hip_stream);
  if (out == nullptr) return MC_ERR_NULL;
  if (!aligned16(out) || !aligned4(lse) || !aligned16(workspace)) return MC_ERR_ALIGN;
  if (workspace == nullptr || workspace_bytes < lay.total) return MC_ERR_WORKSPACE;
  char* ws = reinterpret_cast<char*>(workspace);
  float* o_parts = reinterpret_cast<float*>(ws + lay.o_off);
  float* lse_parts = reinterpret_cast<float*>(ws + lay.lse_off);
  mc_status st = attn_enqueue(p, q, k_pool, v_pool, block_tables, max_pages_per_req, prefix_lens, new_lens, batch,
                              nullptr, nullptr, lay.kv_splits, o_parts, lse_parts, workspace, lay.list_bytes,
                              hip_stream);
  if (st != MC_OK) return st;
  int64_t total_new = 0;
  for (int32_t r = 0; r < batch; ++r) total_new += new_lens[r];
  return mc_attn_merge_lse(o_parts, lse_parts, lay.kv_splits, total_new * p->num_q_heads, p->head_dim, (int32_t)p->dtype,
                           out, lse, hip_stream);
}

mc_status mc_prefill_attn_prepare(const mc_attn_params* p, const int32_t* prefix_lens, const int32_t* new_lens,
                                  int32_t batch, int32_t kv_splits, void* workspace, size_t workspace_bytes,
                                  void* hip_stream, mc_attn_plan* plan) {
  mc_status st = check_params(p);
  if (st != MC_OK) return st;
  if (batch < 0 || kv_splits < 0 || kv_splits > MC_MAX_KV_SPLITS) return MC_ERR_SHAPE;
  if (plan == nullptr || (batch > 0 && (prefix_lens == nullptr || new_lens == nullptr))) return MC_ERR_NULL;
  int64_t total_new = 0;
  int32_t need_pages = 0;
  st = check_lens(p, prefix_lens, new_lens, batch, &total_new, &need_pages);
  if (st != MC_OK) return st;
  if (total_new == 0) {
    // nothing to launch: an empty plan, nothing uploaded
    *plan = mc_attn_plan{0, batch, kv_splits, 0, 0, 0, p->num_q_heads, p->num_kv_heads, (int32_t)p->dtype, 0};
    return MC_OK;
  }
  return prepare_attn(p, prefix_lens, new_lens, batch, kv_splits, total_new, need_pages, workspace, workspace_bytes,
                      reinterpret_cast<hipStream_t>(hip_stream), plan);
}

mc_status mc_prefill_attn_run(const mc_attn_params* p, const mc_attn_plan* plan, const void* q, const void* k_pool,
                              const void* v_pool, const int32_t* block_tables, int32_t max_pages_per_req, void* out,
                              float* lse, const void* workspace, void* hip_stream) {
  mc_status st = check_params(p);
  if (st != MC_OK) return st;
  st = check_plan(p, plan, false);
  if (st != MC_OK) return st;
  if (max_pages_per_req < 0) return MC_ERR_SHAPE;
  if (plan->n_items == 0) return MC_OK;
  st = check_attn_buffers(false, q, k_pool, v_pool, block_tables, plan->batch, max_pages_per_req, plan->need_pages,
                          out, lse, nullptr, nullptr, workspace);
  if (st != MC_OK) return st;
  if (workspace == nullptr) return MC_ERR_WORKSPACE;
  return launch_planned_attn(p, plan, q, k_pool, v_pool, block_tables, max_pages_per_req, out, lse, nullptr, nullptr,
                             workspace, reinterpret_cast<hipStream_t>(hip_stream));
}

mc_status mc_prefill_attn_run_split(const mc_attn_params* p, const mc_attn_plan* plan, const void* q,
                                    const void* k_pool, const void* v_pool, const int32_t* block_tables,
                                    int32_t max_pages_per_req, float* o_parts, float* lse_parts,
                                    const void* workspace, void* hip_stream) {
  mc_status st = check_params(p);
  if (st != MC_OK) return st;
  st = check_plan(p, plan, true);
  if (st != MC_OK) return st;
  if (max_pages_per_req < 0) return MC_ERR_SHAPE;
  if (plan->n_items == 0) return MC_OK;
  st = check_attn_buffers(true, q, k_pool, v_pool, block_tables, plan->batch, max_pages_per_req, plan->need_pages,
                          nullptr, nullptr, o_parts, lse_parts, workspace);
  if (st != MC_OK) return st;
  if (workspace == nullptr) return MC_ERR_WORKSPACE;
  return launch_planned_attn(p, plan, q, k_pool, v_pool, block_tables, max_pages_per_req, nullptr, nullptr, o_parts,
                             lse_parts, workspace, reinterpret_cast<hipStream_t>(hip_stream));
}

mc_status mc_kv_append_run(const mc_attn_params* p, const mc_attn_plan* plan, const void* k_new, const void* v_new,
                           void* k_pool, void* v_pool, const int32_t* block_tables, int32_t max_pages_per_req,
                           const void* workspace, void* hip_stream) {
  mc_status st = check_params(p);
  if (st != MC_OK) return st;
  if (plan == nullptr) return MC_ERR_NULL;
  st = check_plan(p, plan, plan->kv_splits > 0);       // either form of plan holds the request table
  if (st != MC_OK) return st;
  if (max_pages_per_req < 0) return MC_ERR_SHAPE;
  if (plan->n_items == 0) return MC_OK;
  if (max_pages_per_req < plan->need_pages) return MC_ERR_SHAPE;
  if (k_new == nullptr || v_new == nullptr || k_pool == nullptr || v_pool == nullptr || block_tables == nullptr)
    return MC_ERR_NULL;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(workspace) ||
      !aligned4(block_tables))
    return MC_ERR_ALIGN;
  const int64_t total_new = plan->total_new_tokens;
  if (total_new > INT32_MAX || total_new * p->num_kv_heads * 16 / 256 + 1 > INT32_MAX ||
      (int64_t)plan->batch * max_pages_per_req > INT32_MAX)
    return MC_ERR_RANGE;
  if (workspace == nullptr) return MC_ERR_WORKSPACE;
  const char* ws = reinterpret_cast<const char*>(workspace);
  if (mc::launch_kv_append(k_new, v_new, k_pool, v_pool, block_tables, max_pages_per_req,
                           reinterpret_cast<const mc::AttnReq*>(ws + plan->reqs_offset), plan->batch, total_new,
                           p->num_kv_heads, row_bytes_of(p), reinterpret_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return MC_ERR_HIP;
  return MC_OK;
}

mc_status mc_prefill_attn_plan(const mc_attn_params* p, const int32_t* prefix_lens, const int32_t* new_lens,
                               int32_t batch, int32_t kv_splits, int32_t* items, int64_t capacity,
                               int64_t* n_items) {
  return plan_items(p, prefix_lens, new_lens, batch, kv_splits, items, capacity, n_items);
}

int32_t mc_prefill_attn_suggest_kv_splits(const mc_attn_params* p, const int32_t* prefix_lens,
                                          const int32_t* new_lens, int32_t batch) {
  return suggest_kv_splits(p, prefix_lens, new_lens, batch);
}

mc_status mc_attn_merge_lse(const float* o_parts, const float* lse_parts, int32_t kv_splits, int64_t rows,
                            int32_t head_dim, int32_t dtype, void* out, float* lse, void* hip_stream) {
  if (kv_splits < 1 || kv_splits > MC_MAX_KV_SPLITS || rows < 0 || head_dim <= 0) return MC_ERR_SHAPE;
  if (!((dtype == MC_DTYPE_BF16 && (head_dim == 128 || head_dim == 64)) || (dtype == MC_DTYPE_F32 && head_dim == 64)))
    return MC_ERR_UNSUPPORTED;
  if (rows == 0) return MC_OK;
  if (o_parts == nullptr || lse_parts == nullptr || out == nullptr) return MC_ERR_NULL;
  if (!aligned16(o_parts) || !aligned16(out) || !aligned4(lse_parts) ||
      !aligned4(lse))
    return MC_ERR_ALIGN;
  if (rows > INT32_MAX) return MC_ERR_RANGE;
  if (mc::launch_attn_merge(dtype, head_dim, o_parts, lse_parts, kv_splits, rows, out, lse,
                            reinterpret_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return MC_ERR_HIP;
  return MC_OK;
}

size_t mc_kv_append_workspace_bytes(int32_t batch) {
  return batch < 0 ? 0 : sizeof(mc::AttnReq) * (size_t)batch + 64;
}

mc_status mc_kv_append_paged(const mc_attn_params* p, const void* k_new, const void* v_new, void* k_pool,
                             void* v_pool, const int32_t* block_tables, int32_t max_pages_per_req,
                             const int32_t* prefix_lens, const int32_t* new_lens, int32_t batch,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
  mc_status st = check_params(p);
  if (st != MC_OK) return st;
  if (batch < 0 || max_pages_per_req < 0) return MC_ERR_SHAPE;
  if (batch == 0) return MC_OK;
  if (prefix_lens == nullptr || new_lens == nullptr) return MC_ERR_NULL;
  int64_t total_new = 0;
  for (int32_t r = 0; r < batch; ++r) {
    if (prefix_lens[r] < 0 || new_lens[r] < 0) return MC_ERR_SHAPE;
    const int64_t len = (int64_t)prefix_lens[r] + new_lens[r];
    if (len > INT32_MAX - 1024) return MC_ERR_RANGE;
    if (new_lens[r] > 0 && (int64_t)max_pages_per_req * p->page_size < len) return MC_ERR_SHAPE;
    total_new += new_lens[r];
  }
  if (total_new == 0) return MC_OK;
  if (k_new == nullptr || v_new == nullptr || k_pool == nullptr || v_pool == nullptr || block_tables == nullptr)
    return MC_ERR_NULL;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(workspace) ||
      !aligned4(block_tables))
    return MC_ERR_ALIGN;
  if (total_new > INT32_MAX || total_new * p->num_kv_heads * 16 / 256 + 1 > INT32_MAX ||
      (int64_t)batch * max_pages_per_req > INT32_MAX)
    return MC_ERR_RANGE;
  if (workspace == nullptr || workspace_bytes < mc_kv_append_workspace_bytes(batch)) return MC_ERR_WORKSPACE;

  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const size_t up_bytes = sizeof(mc::AttnReq) * (size_t)batch;
  int slot = -1;
  mc::AttnReq* host = reinterpret_cast<mc::AttnReq*>(g_staging.acquire(up_bytes, &slot));
  if (host == nullptr) return MC_ERR_HIP;
  int64_t q_off = 0;
  for (int32_t r = 0; r < batch; ++r) {
    host[r] = {(int32_t)q_off, prefix_lens[r], new_lens[r],
               (int32_t)(((int64_t)prefix_lens[r] + new_lens[r] + p->page_size - 1) / p->page_size)};
    q_off += new_lens[r];
  }
  if (hipMemcpyAsync(workspace, host, up_bytes, hipMemcpyHostToDevice, stream) != hipSuccess) {
    g_staging.abandon(slot);
    return MC_ERR_HIP;
  }
  if (!g_staging.release_after(slot, stream)) return MC_ERR_HIP;
  if (mc::launch_kv_append(k_new, v_new, k_pool, v_pool, block_tables, max_pages_per_req,
                           reinterpret_cast<const mc::AttnReq*>(workspace), batch, total_new, p->num_kv_heads,
                           row_bytes_of(p), stream) != hipSuccess)
    return MC_ERR_HIP;
  return MC_OK;
}

mc_status mc_kv_page_order(const int32_t* page_ids, int64_t n, int32_t* order, void* hip_stream) {
  if (n < 0) return MC_ERR_SHAPE;
  if (n == 0) return MC_OK;
  if (page_ids == nullptr || order == nullptr) return MC_ERR_NULL;
  if (!aligned4(page_ids) || !aligned4(order)) return MC_ERR_ALIGN;
  if (n > (int64_t)1 << 20) return MC_ERR_RANGE;   // quadratic in n: a request's page list, not a pool
  if (mc::launch_kv_page_order(page_ids, n, order, reinterpret_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return MC_ERR_HIP;
  return MC_OK;
}

mc_status mc_kv_check_page_ids(const int32_t* page_ids, int64_t n, int64_t num_pages, int32_t* report,
                               void* hip_stream) {
  if (n < 0 || num_pages < 0) return MC_ERR_SHAPE;
  if (n == 0) return MC_OK;
  if (page_ids == nullptr || report == nullptr) return MC_ERR_NULL;
  if (!aligned4(page_ids) || !aligned4(report)) return MC_ERR_ALIGN;
  if (n > INT32_MAX) return MC_ERR_RANGE;
  if (mc::launch_kv_check_page_ids(page_ids, n, num_pages, report, reinterpret_cast<hipStream_t>(hip_stream)) !=
      hipSuccess)
    return MC_ERR_HIP;
  return MC_OK;
}

mc_status mc_kv_pack_layer_ordered(const void* k_pool_layer, const void* v_pool_layer, int64_t num_pages,
                                   int64_t page_bytes, const int32_t* page_ids, const int32_t* order, int64_t n,
                                   void* k_out, void* v_out, void* hip_stream) {
  mc_status st = check_copy(k_pool_layer, v_pool_layer, num_pages, page_bytes, page_ids, n, k_out, v_out);
  if (st != MC_OK || n == 0 || page_bytes == 0) return st;
  if (!aligned4(order)) return MC_ERR_ALIGN;
  if (mc::launch_kv_copy(true, k_pool_layer, v_pool_layer, k_out, v_out, page_ids, order, n, page_bytes,
                         reinterpret_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return MC_ERR_HIP;
  return MC_OK;
}

mc_status mc_kv_unpack_layer_ordered(const void* k_in, const void* v_in, int64_t num_pages, int64_t page_bytes,
                                     const int32_t* page_ids, const int32_t* order, int64_t n, void* k_pool_layer,
                                     void* v_pool_layer, void* hip_stream) {
  mc_status st = check_copy(k_in, v_in, num_pages, page_bytes, page_ids, n, k_pool_layer, v_pool_layer);
  if (st != MC_OK || n == 0 || page_bytes == 0) return st;
  if (!aligned4(order)) return MC_ERR_ALIGN;
  if (mc::launch_kv_copy(false, k_in, v_in, k_pool_layer, v_pool_layer, page_ids, order, n, page_bytes,
                         reinterpret_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return MC_ERR_HIP;
  return MC_OK;
}

mc_status mc_kv_pack_layer(const void* k_pool_layer, const void* v_pool_layer, int64_t num_pages, int64_t page_bytes,
                           const int32_t* page_ids, int64_t n, void* k_out, void* v_out, void* hip_stream) {
  return mc_kv_pack_layer_ordered(k_pool_layer, v_pool_layer, num_pages, page_bytes, page_ids, nullptr, n, k_out,
                                  v_out, hip_stream);
}

mc_status mc_kv_unpack_layer(const void* k_in, const void* v_in, int64_t num_pages, int64_t page_bytes,
                             const int32_t* page_ids, int64_t n, void* k_pool_layer, void* v_pool_layer,
                             void* hip_stream) {
  return mc_kv_unpack_layer_ordered(k_in, v_in, num_pages, page_bytes, page_ids, nullptr, n, k_pool_layer,
                                    v_pool_layer, hip_stream);
}

mc_status mc_kv_load_layer(const void* k_host, const void* v_host, void* k_stage, void* v_stage, int64_t num_pages,
                           int64_t page_bytes, const int32_t* page_ids, int64_t n, void* k_pool_layer,
                           void* v_pool_layer, void* hip_stream) {
  mc_status st = check_copy(k_stage, v_stage, num_pages, page_bytes, page_ids, n, k_pool_layer, v_pool_layer);
  if (st != MC_OK || n == 0 || page_bytes == 0) return st;
  if (k_host == nullptr || v_host == nullptr) return MC_ERR_NULL;
  if (!aligned16(k_host) || !aligned16(v_host)) return MC_ERR_ALIGN;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const size_t bytes = (size_t)n * (size_t)page_bytes;
  if (hipMemcpyAsync(k_stage, k_host, bytes, hipMemcpyHostToDevice, stream) != hipSuccess) return MC_ERR_HIP;
  if (hipMemcpyAsync(v_stage, v_host, bytes, hipMemcpyHostToDevice, stream) != hipSuccess) return MC_ERR_HIP;
  if (mc::launch_kv_copy(false, k_stage, v_stage, k_pool_layer, v_pool_layer, page_ids, nullptr, n, page_bytes, stream) !=
      hipSuccess)
    return MC_ERR_HIP;
  return MC_OK;
}

mc_status mc_kv_store_layer(const void* k_pool_layer, const void* v_pool_layer, int64_t num_pages,
                            int64_t page_bytes, const int32_t* page_ids, int64_t n, void* k_stage, void* v_stage,
                            void* k_host, void* v_host, void* hip_stream) {
  mc_status st = check_copy(k_pool_layer, v_pool_layer, num_pages, page_bytes, page_ids, n, k_stage, v_stage);
  if (st != MC_OK || n == 0 || page_bytes == 0) return st;
  if (k_host == nullptr || v_host == nullptr) return MC_ERR_NULL;
  if (!aligned16(k_host) || !aligned16(v_host)) return MC_ERR_ALIGN;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const size_t bytes = (size_t)n * (size_t)page_bytes;
  if (mc::launch_kv_copy(true, k_pool_layer, v_pool_layer, k_stage, v_stage, page_ids, nullptr, n, page_bytes, stream) !=
      hipSuccess)
    return MC_ERR_HIP;
  if (hipMemcpyAsync(k_host, k_stage, bytes, hipMemcpyDeviceToHost, stream) != hipSuccess) return MC_ERR_HIP;
  if (hipMemcpyAsync(v_host, v_stage, bytes, hipMemcpyDeviceToHost, stream) != hipSuccess) return MC_ERR_HIP;
  return MC_OK;
}


size_t mc_prefix_hash_workspace_bytes(int32_t batch) {
  return batch < 0 ? 0 : 2 * sizeof(int64_t) * ((size_t)batch + 1) + 64;
}

mc_status mc_prefix_hash(const int32_t* tokens, const int64_t* tok_offsets, int32_t batch, int32_t block_tokens,
                         uint64_t* keys, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (batch < 0 || block_tokens <= 0) return MC_ERR_SHAPE;
  if (batch == 0) return MC_OK;
  if (tok_offsets == nullptr) return MC_ERR_NULL;
  std::vector<int64_t> tab(2 * ((size_t)batch + 1));
  int64_t* key_off = tab.data() + batch + 1;
  key_off[0] = 0;
  int64_t max_blocks = 0;
  for (int32_t r = 0; r < batch; ++r) {
    const int64_t len = tok_offsets[r + 1] - tok_offsets[r];
    if (len < 0 || tok_offsets[r] < 0) return MC_ERR_SHAPE;
    const int64_t blocks = (len + block_tokens - 1) / block_tokens;
    key_off[r + 1] = key_off[r] + blocks;
    max_blocks = blocks > max_blocks ? blocks : max_blocks;
  }
  const int64_t total_blocks = key_off[batch];
  if (total_blocks == 0) return MC_OK;
  if (tokens == nullptr || keys == nullptr) return MC_ERR_NULL;
  if (!aligned4(tokens) || (reinterpret_cast<uintptr_t>(keys) & 7u) ||
      !aligned16(workspace))
    return MC_ERR_ALIGN;
  if (max_blocks > (1 << 26) - 8) return MC_ERR_RANGE;   // four blocks per workgroup along grid x
  if (workspace == nullptr || workspace_bytes < mc_prefix_hash_workspace_bytes(batch)) return MC_ERR_WORKSPACE;
  std::memcpy(tab.data(), tok_offsets, sizeof(int64_t) * ((size_t)batch + 1));
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const size_t up = sizeof(int64_t) * tab.size();
  int slot = -1;
  void* host = g_staging.acquire(up, &slot);
  if (host == nullptr) return MC_ERR_HIP;
  std::memcpy(host, tab.data(), up);
  if (hipMemcpyAsync(workspace, host, up, hipMemcpyHostToDevice, stream) != hipSuccess) {
    g_staging.abandon(slot);
    return MC_ERR_HIP;
  }
  if (!g_staging.release_after(slot, stream)) return MC_ERR_HIP;
  const int64_t* dev_tab = reinterpret_cast<const int64_t*>(workspace);
  if (mc::launch_prefix_hash(tokens, dev_tab, dev_tab + batch + 1, batch, block_tokens, max_blocks, keys, stream) !=
      hipSuccess)
    return MC_ERR_HIP;
  return MC_OK;
}

size_t mc_prefix_match_workspace_bytes(int32_t batch, int32_t n_inst) {
  return (batch < 0 || n_inst < 0) ? 0 : sizeof(int64_t) * ((size_t)batch + 1 + (size_t)n_inst + 1) + 64;
}

mc_status mc_prefix_match(const uint64_t* keys, const int64_t* key_offsets, int32_t batch, const uint64_t* cache_keys,
                          const int64_t* cache_offsets, int32_t n_inst, int32_t* prefix_len, int32_t* best_len,
                          int32_t* best_inst, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (batch < 0 || n_inst < 0) return MC_ERR_SHAPE;
  if (batch == 0) return MC_OK;
  if (key_offsets == nullptr || cache_offsets == nullptr) return MC_ERR_NULL;
  if (key_offsets[0] < 0 || cache_offsets[0] < 0) return MC_ERR_SHAPE;
  for (int32_t r = 0; r < batch; ++r) {
    if (key_offsets[r + 1] < key_offsets[r]) return MC_ERR_SHAPE;
    if (key_offsets[r + 1] - key_offsets[r] > INT32_MAX) return MC_ERR_RANGE;
  }
  for (int32_t i = 0; i < n_inst; ++i)
    if (cache_offsets[i + 1] < cache_offsets[i]) return MC_ERR_SHAPE;
  if (best_len == nullptr || best_inst == nullptr || (n_inst > 0 && prefix_len == nullptr)) return MC_ERR_NULL;
  if ((key_offsets[batch] > key_offsets[0] && keys == nullptr) ||
      (cache_offsets[n_inst] > cache_offsets[0] && cache_keys == nullptr))
    return MC_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(keys) & 7u) || (reinterpret_cast<uintptr_t>(cache_keys) & 7u) ||
      !aligned4(prefix_len) || !aligned4(best_len) ||
      !aligned4(best_inst) || !aligned16(workspace))
    return MC_ERR_ALIGN;
  if (batch > 65535) return MC_ERR_RANGE;   // the match grid's second dimension
  if (workspace == nullptr || workspace_bytes < mc_prefix_match_workspace_bytes(batch, n_inst)) return MC_ERR_WORKSPACE;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const size_t n_tab = (size_t)batch + 1 + (size_t)n_inst + 1;
  const size_t up = sizeof(int64_t) * n_tab;
  int slot = -1;
  int64_t* host = reinterpret_cast<int64_t*>(g_staging.acquire(up, &slot));
  if (host == nullptr) return MC_ERR_HIP;
  std::memcpy(host, key_offsets, sizeof(int64_t) * ((size_t)batch + 1));
  std::memcpy(host + batch + 1, cache_offsets, sizeof(int64_t) * ((size_t)n_inst + 1));
  if (hipMemcpyAsync(workspace, host, up, hipMemcpyHostToDevice, stream) != hipSuccess) {
    g_staging.abandon(slot);
    return MC_ERR_HIP;
  }
  if (!g_staging.release_after(slot, stream)) return MC_ERR_HIP;
  const int64_t* dev_tab = reinterpret_cast<const int64_t*>(workspace);
  if (mc::launch_prefix_match(keys, dev_tab, batch, cache_keys, dev_tab + batch + 1, n_inst, prefix_len, best_len,
                              best_inst, stream) != hipSuccess)
    return MC_ERR_HIP;
  return MC_OK;
}

}  // extern "C"
