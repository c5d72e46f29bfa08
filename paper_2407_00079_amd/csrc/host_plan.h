// Host-side half of the C-ABI front end: argument validation, the attention work list, the
// key-slice suggestion, workspace layouts and the bookkeeping of the pinned staging slots.
// Nothing here calls HIP, so the file also builds with a plain host compiler and its
// sanitizers (tests do that).
#pragma once
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "mc.h"
#include "mc_types.h"

namespace mc {
namespace host {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

mc_status check_params(const mc_attn_params* p);

// softmax scale (0 selects 1 / sqrt(head_dim)) times log2(e): the kernels form probabilities with exp2
float attn_scale_log2e(const mc_attn_params* p);

// upper bound on work items: per request and KV head, ceil(C_r * G / rows) <= C_r * G / rows + 1
size_t max_items(const mc_attn_params* p, int32_t batch, int64_t total_new_tokens, int32_t kv_splits = 1);

// bytes of work list + request table for that bound (what the *_workspace_bytes calls return)
size_t list_bytes(const mc_attn_params* p, int32_t batch, int64_t total_new_tokens, int32_t kv_splits = 1);

// Lengths of a batch: sign and range checks, sum of the new tokens, most pages any request
// with new tokens needs.
mc_status check_lens(const mc_attn_params* p, const int32_t* prefix_lens, const int32_t* new_lens, int32_t batch,
                     int64_t* total_new, int32_t* need_pages);

// Everything an attention launch checks besides the lengths.  split == false: the whole-row kernel
// writes out / lse.  split == true: the split kernel writes partials (out / lse unused).
mc_status check_attn_buffers(bool split, const void* q, const void* k_pool, const void* v_pool,
                             const int32_t* block_tables, int32_t batch, int32_t max_pages_per_req, int32_t need_pages,
                             const void* out, const float* lse, const float* o_parts, const float* lse_parts,
                             const void* workspace);

// sizes that must hold before a work list is built: row and item counts the kernels index with 32 bits
mc_status check_list_range(const mc_attn_params* p, int32_t batch, int64_t total_new, int32_t kv_splits);

// Work list of an attention launch: one item per (request, KV head, tile of stacked rows) and, for
// split launches (kv_splits >= 1), per key slice - most keys first, dealt round-robin so that
// consecutive workgroup ids (which land on different XCDs) take different (request, KV head)
// streams and each XCD's L2 keeps one stream hot.  Lengths have been validated by the caller.
void build_work_list(const mc_attn_params* p, const int32_t* prefix_lens, const int32_t* new_lens, int32_t batch,
                     int32_t kv_splits, std::vector<AttnReq>& reqs, std::vector<AttnItem>& items);

// number of whole-row work items of a batch (the size of the list build_work_list makes for kv_splits == 0)
int64_t count_items(const mc_attn_params* p, const int32_t* new_lens, int32_t batch);

// A plan handed back by the caller: made for these params, of the wanted form, not empty.
mc_status check_plan(const mc_attn_params* p, const mc_attn_plan* plan, bool want_split);

// the body of mc_prefill_attn_plan and of mc_prefill_attn_suggest_kv_splits
mc_status plan_items(const mc_attn_params* p, const int32_t* prefix_lens, const int32_t* new_lens, int32_t batch,
                     int32_t kv_splits, int32_t* items, int64_t capacity, int64_t* n_items);
int32_t suggest_kv_splits(const mc_attn_params* p, const int32_t* prefix_lens, const int32_t* new_lens,
                          int32_t batch);

// Workspace of the automatic form: [work list + request table | o_parts | lse_parts], each part
// starting at a multiple of 256 bytes.
struct AutoLayout {
  int32_t kv_splits;
  size_t list_bytes, o_off, lse_off, total;
};
bool auto_layout(const mc_attn_params* p, const int32_t* prefix_lens, const int32_t* new_lens, int32_t batch,
                 AutoLayout* lay);

// arguments of a page copy (pack / unpack and their relatives): a, b source pair, c, d destination pair
mc_status check_copy(const void* a, const void* b, int64_t num_pages, int64_t page_bytes, const int32_t* ids,
                     int64_t n, const void* c, const void* d);

// Bookkeeping of the pinned host slots that work lists and tables are written to before their
// asynchronous upload.  A slot is FREE, HELD by a call that is filling it (between acquire and
// the event recorded behind its upload), or IN FLIGHT (its event decides when it is free again).
// A held slot is never handed out, whichever thread asks: the state is set under the owner's
// lock when the slot is picked, not when the upload has been enqueued.  The events and the
// memory themselves belong to the owner; this class only decides which slot a call gets.
class SlotRing {
 public:
  static constexpr int kMaxSlots = 256;
  enum State : int { kFree = 0, kHeld = 1, kInFlight = 2 };
  struct Pick {
    int slot;        // index, or -1: the ring is full of held slots or of other devices' slots
    bool is_new;     // the owner has to create the slot's event (and memory) first
    bool must_wait;  // every slot of the device is in flight and the ring is full: wait for this one's event
  };
  // `done(i)` tells whether the event of in-flight slot i has completed.  The returned slot is HELD.
  template <class Done>
  Pick pick(int dev, Done&& done) {
    const int n = n_;
    for (int k = 0; k < n; ++k) {
      const int i = (next_ + k) % n;
      if (dev_[i] != dev || state_[i] == kHeld) continue;
      if (state_[i] == kFree || done(i)) return take(i, false, false);
    }
    if (n < kMaxSlots) {
      dev_[n] = dev;
      ++n_;
      return take(n, true, false);
    }
    for (int k = 0; k < n; ++k) {
      const int i = (next_ + k) % n;
      if (dev_[i] == dev && state_[i] == kInFlight) return take(i, false, true);
    }
    return Pick{-1, false, false};
  }
  // the upload from the slot has been enqueued and its event recorded
  void in_flight(int slot) { state_[slot] = kInFlight; }
  // the call gave up before anything was enqueued from the slot (or its event could not be recorded
  // and the owner has waited for the stream instead)
  void abandon(int slot) { state_[slot] = kFree; }
  // a new slot whose event could not be created is taken out again (it is the last one)
  void drop_new(int slot) {
    if (slot == n_ - 1) --n_;
    else state_[slot] = kFree;
  }
  int size() const { return n_; }
  State state(int slot) const { return (State)state_[slot]; }
  int device(int slot) const { return dev_[slot]; }

 private:
  Pick take(int i, bool is_new, bool must_wait) {
    state_[i] = kHeld;
    next_ = (i + 1) % n_;
    return Pick{i, is_new, must_wait};
  }
  int n_ = 0, next_ = 0;
  int dev_[kMaxSlots] = {};
  int state_[kMaxSlots] = {};
};

}  // namespace host
}  // namespace mc
