// Native driver for the host-side planning code (csrc/host_plan.cpp), built by
// tests/test_host_sanitized.py with g++ -fsanitize=address,undefined.  No GPU, no HIP.
//
//   host_plan_driver selftest          rejection cases and the staging-slot state machine; exit 0 = pass
//   host_plan_driver plan < requests   one line per request:
//       Hq Hkv head_dim dtype kv_splits batch P_0 C_0 P_1 C_1 ...
//     answers "status n_items suggested_splits list_bytes" and then one line "req head row0 slice" per item
#include <cstdio>
#include <cstdlib>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "host_plan.h"

using namespace mc::host;

static int failures = 0;
#define EXPECT(cond)                                                        \
  do {                                                                      \
    if (!(cond)) {                                                          \
      std::fprintf(stderr, "line %d: EXPECT(%s) failed\n", __LINE__, #cond); \
      ++failures;                                                           \
    }                                                                       \
  } while (0)

static mc_attn_params good() { return mc_attn_params{64, 8, 128, 16, 4096, MC_DTYPE_BF16, 0.f}; }
static const void* const FAKE = reinterpret_cast<const void*>(0x7F0000001000ull);
static const void* off(const void* p, int by) { return reinterpret_cast<const char*>(p) + by; }

static void test_rejections() {
  mc_attn_params p = good();
  EXPECT(check_params(nullptr) == MC_ERR_NULL);
  EXPECT(check_params(&p) == MC_OK);
  p = good(); p.num_kv_heads = 7;  EXPECT(check_params(&p) == MC_ERR_SHAPE);
  p = good(); p.head_dim = 96;     EXPECT(check_params(&p) == MC_ERR_UNSUPPORTED);
  p = good(); p.page_size = 32;    EXPECT(check_params(&p) == MC_ERR_UNSUPPORTED);
  p = good(); p.dtype = 5;         EXPECT(check_params(&p) == MC_ERR_UNSUPPORTED);
  p = good(); p.dtype = MC_DTYPE_F32; EXPECT(check_params(&p) == MC_ERR_UNSUPPORTED);   // f32 needs head_dim 64
  p = good(); p.softmax_scale = -1.f; EXPECT(check_params(&p) == MC_ERR_SHAPE);
  p = good(); p.num_pages = 0;     EXPECT(check_params(&p) == MC_ERR_SHAPE);

  p = good();
  int64_t total = 0;
  int32_t pages = 0;
  {
    const int32_t P[2] = {100, 7}, C[2] = {33, 0};
    EXPECT(check_lens(&p, P, C, 2, &total, &pages) == MC_OK && total == 33 && pages == 9);
    const int32_t N[1] = {-1};
    EXPECT(check_lens(&p, N, C, 1, &total, &pages) == MC_ERR_SHAPE);
    EXPECT(check_lens(&p, P, N, 1, &total, &pages) == MC_ERR_SHAPE);
    const int32_t big[1] = {INT32_MAX - 8}, sixteen[1] = {16};
    EXPECT(check_lens(&p, big, sixteen, 1, &total, &pages) == MC_ERR_RANGE);
    EXPECT(check_lens(&p, nullptr, nullptr, 0, &total, &pages) == MC_OK && total == 0 && pages == 0);
  }
  const int32_t* bt = reinterpret_cast<const int32_t*>(FAKE);
  const float* nof = nullptr;
  EXPECT(check_attn_buffers(false, FAKE, FAKE, FAKE, bt, 1, 1024, 1024, FAKE, nof, nof, nof, FAKE) == MC_OK);
  EXPECT(check_attn_buffers(false, FAKE, FAKE, FAKE, bt, 1, 1023, 1024, FAKE, nof, nof, nof, FAKE) == MC_ERR_SHAPE);
  EXPECT(check_attn_buffers(false, nullptr, FAKE, FAKE, bt, 1, 1024, 1024, FAKE, nof, nof, nof, FAKE) == MC_ERR_NULL);
  EXPECT(check_attn_buffers(false, FAKE, FAKE, FAKE, nullptr, 1, 1024, 1024, FAKE, nof, nof, nof, FAKE) == MC_ERR_NULL);
  EXPECT(check_attn_buffers(false, FAKE, FAKE, FAKE, bt, 1, 1024, 1024, nullptr, nof, nof, nof, FAKE) == MC_ERR_NULL);
  EXPECT(check_attn_buffers(false, off(FAKE, 8), FAKE, FAKE, bt, 1, 1024, 1024, FAKE, nof, nof, nof, FAKE) == MC_ERR_ALIGN);
  EXPECT(check_attn_buffers(false, FAKE, off(FAKE, 2), FAKE, bt, 1, 1024, 1024, FAKE, nof, nof, nof, FAKE) == MC_ERR_ALIGN);
  EXPECT(check_attn_buffers(false, FAKE, FAKE, FAKE, bt, 1, 1024, 1024, FAKE, reinterpret_cast<const float*>(off(FAKE, 2)), nof,
                            nof, FAKE) == MC_ERR_ALIGN);
  EXPECT(check_attn_buffers(true, FAKE, FAKE, FAKE, bt, 1, 1024, 1024, nullptr, nof, nof, nof, FAKE) == MC_ERR_NULL);
  EXPECT(check_attn_buffers(true, FAKE, FAKE, FAKE, bt, 1, 1024, 1024, nullptr, nof, reinterpret_cast<const float*>(FAKE),
                            reinterpret_cast<const float*>(FAKE), FAKE) == MC_OK);
  EXPECT(check_attn_buffers(false, FAKE, FAKE, FAKE, bt, 70000, 70000, 10, FAKE, nof, nof, nof, FAKE) == MC_ERR_RANGE);

  const int32_t* ids = reinterpret_cast<const int32_t*>(FAKE);
  EXPECT(check_copy(FAKE, FAKE, 64, 4096, ids, 24, FAKE, FAKE) == MC_OK);
  EXPECT(check_copy(nullptr, FAKE, 64, 4096, ids, 24, FAKE, FAKE) == MC_ERR_NULL);
  EXPECT(check_copy(FAKE, FAKE, 64, 4096, ids, 24, FAKE, nullptr) == MC_ERR_NULL);
  EXPECT(check_copy(FAKE, FAKE, 64, 4096, nullptr, 24, FAKE, FAKE) == MC_ERR_NULL);
  EXPECT(check_copy(FAKE, FAKE, 64, 4100, ids, 24, FAKE, FAKE) == MC_ERR_ALIGN);
  EXPECT(check_copy(FAKE, off(FAKE, 4), 64, 4096, ids, 24, FAKE, FAKE) == MC_ERR_ALIGN);
  EXPECT(check_copy(FAKE, FAKE, 64, 4096, ids, -1, FAKE, FAKE) == MC_ERR_SHAPE);
  EXPECT(check_copy(FAKE, FAKE, 64, -16, ids, 24, FAKE, FAKE) == MC_ERR_SHAPE);
  EXPECT(check_copy(FAKE, FAKE, 0, 4096, ids, 24, FAKE, FAKE) == MC_ERR_SHAPE);
  EXPECT(check_copy(FAKE, FAKE, 64, 4096, ids, (int64_t)1 << 31, FAKE, FAKE) == MC_ERR_RANGE);
  EXPECT(check_copy(FAKE, FAKE, 64, 32768, ids, (int64_t)1 << 30, FAKE, FAKE) == MC_ERR_RANGE);   // 4 slices per page
  EXPECT(check_copy(nullptr, nullptr, 64, 4096, nullptr, 0, nullptr, nullptr) == MC_OK);

  mc_attn_plan plan{2048, 1, 0, 1024, 8192, 32768, 64, 8, MC_DTYPE_BF16, 0};
  EXPECT(check_plan(&p, &plan, false) == MC_OK);
  EXPECT(check_plan(&p, &plan, true) == MC_ERR_SHAPE);
  EXPECT(check_plan(&p, nullptr, false) == MC_ERR_NULL);
  mc_attn_params other = good();
  other.num_q_heads = 32;
  EXPECT(check_plan(&other, &plan, false) == MC_ERR_SHAPE);
  plan.reqs_offset = 8;
  EXPECT(check_plan(&p, &plan, false) == MC_ERR_SHAPE);

  int64_t n = -1;
  const int32_t P1[1] = {8192}, C1[1] = {8192};
  EXPECT(plan_items(&p, P1, C1, 1, 0, nullptr, 0, &n) == MC_OK && n == 2048);
  std::vector<int32_t> small(40, -5);
  EXPECT(plan_items(&p, P1, C1, 1, 0, small.data(), 10, &n) == MC_ERR_WORKSPACE && n == 2048);
  for (int32_t v : small) EXPECT(v == -5);
  EXPECT(plan_items(&p, P1, C1, 1, 0, nullptr, 0, nullptr) == MC_ERR_NULL);
  EXPECT(plan_items(&p, P1, C1, 1, MC_MAX_KV_SPLITS + 1, nullptr, 0, &n) == MC_ERR_SHAPE);
  EXPECT(count_items(&p, C1, 1) == 2048);
  EXPECT(list_bytes(&p, 1, 8192) >= 16u * 2048 + 16);
  AutoLayout lay;
  const int32_t P2[1] = {131056}, C2[1] = {16};
  EXPECT(auto_layout(&p, P2, C2, 1, &lay) && lay.kv_splits == 32 && lay.o_off % 256 == 0 && lay.lse_off % 256 == 0 &&
         lay.total == lay.lse_off + (size_t)32 * 16 * 64 * 4);
  const int32_t neg[1] = {-1};
  EXPECT(!auto_layout(&p, neg, C2, 1, &lay));
}

// The slot bookkeeping, driven the way the staging ring drives it: `done` stands in for hipEventQuery.
static void test_slot_ring() {
  SlotRing ring;
  std::vector<char> finished(SlotRing::kMaxSlots, 0);
  auto done = [&](int i) { return finished[i] != 0; };
  // two acquires with nothing released in between must never share a slot (the reported race:
  // a slot used to count as free until its upload had been enqueued)
  SlotRing::Pick a = ring.pick(0, done), b = ring.pick(0, done);
  EXPECT(a.slot >= 0 && b.slot >= 0 && a.slot != b.slot && a.is_new && b.is_new && !a.must_wait);
  EXPECT(ring.state(a.slot) == SlotRing::kHeld && ring.state(b.slot) == SlotRing::kHeld);
  // a upload enqueued, not finished: a third call gets a third slot
  ring.in_flight(a.slot);
  SlotRing::Pick c = ring.pick(0, done);
  EXPECT(c.slot != a.slot && c.slot != b.slot && c.is_new);
  // a finished: the next call takes it back, and it is held again
  finished[a.slot] = 1;
  ring.in_flight(c.slot);
  SlotRing::Pick d = ring.pick(0, done);
  EXPECT(d.slot == a.slot && !d.is_new && !d.must_wait && ring.state(a.slot) == SlotRing::kHeld);
  finished[a.slot] = 0;
  // a call that gives up frees its slot without an event
  ring.abandon(b.slot);
  SlotRing::Pick e = ring.pick(0, done);
  EXPECT(e.slot == b.slot && !e.is_new);
  // another device never gets this device's slots
  SlotRing::Pick f = ring.pick(1, done);
  EXPECT(f.is_new && ring.device(f.slot) == 1);
  ring.abandon(f.slot);
  SlotRing::Pick g = ring.pick(1, done);
  EXPECT(g.slot == f.slot && !g.is_new);
  // a slot whose event could not be created is taken out again
  const int before = ring.size();
  SlotRing::Pick h = ring.pick(2, done);
  EXPECT(h.is_new && ring.size() == before + 1);
  ring.drop_new(h.slot);
  EXPECT(ring.size() == before);

  // full ring: everything in flight -> the oldest is waited for; everything held -> refusal
  SlotRing full;
  for (int i = 0; i < SlotRing::kMaxSlots; ++i) {
    SlotRing::Pick p = full.pick(0, done);
    EXPECT(p.slot == i && p.is_new);
  }
  EXPECT(full.pick(0, done).slot == -1);            // all held by calls that are still filling them
  for (int i = 0; i < SlotRing::kMaxSlots; ++i) full.in_flight(i);
  std::fill(finished.begin(), finished.end(), 0);
  SlotRing::Pick w = full.pick(0, done);
  EXPECT(w.slot >= 0 && w.must_wait && !w.is_new && full.state(w.slot) == SlotRing::kHeld);
  SlotRing::Pick w2 = full.pick(0, done);
  EXPECT(w2.slot >= 0 && w2.slot != w.slot && w2.must_wait);
  EXPECT(full.pick(1, done).slot == -1);            // no room for another device's slot

  // two threads acquiring and releasing under one lock, as the library does: a slot is never
  // owned twice at a time
  SlotRing shared;
  std::mutex mu;
  std::vector<int> owner(SlotRing::kMaxSlots, 0);
  std::vector<char> fin(SlotRing::kMaxSlots, 1);
  int clashes = 0;
  auto worker = [&](int id) {
    for (int it = 0; it < 20000; ++it) {
      int slot;
      {
        std::lock_guard<std::mutex> lock(mu);
        slot = shared.pick(0, [&](int i) { return fin[i] != 0; }).slot;
        if (slot < 0) continue;
        if (owner[slot] != 0) ++clashes;
        owner[slot] = id;
      }
      // ... the call fills the slot here, outside the lock ...
      {
        std::lock_guard<std::mutex> lock(mu);
        if (owner[slot] != id) ++clashes;
        owner[slot] = 0;
        if (it % 7 == 0) shared.abandon(slot);
        else shared.in_flight(slot);
      }
    }
  };
  std::thread t1(worker, 1), t2(worker, 2), t3(worker, 3);
  t1.join();
  t2.join();
  t3.join();
  EXPECT(clashes == 0);
  EXPECT(shared.size() <= 3);
}

static int run_plans() {
  for (;;) {
    int Hq, Hkv, D, dtype, kv_splits, batch;
    if (std::scanf("%d %d %d %d %d %d", &Hq, &Hkv, &D, &dtype, &kv_splits, &batch) != 6) return 0;
    std::vector<int32_t> P((size_t)(batch > 0 ? batch : 0)), C(P.size());
    for (size_t r = 0; r < P.size(); ++r)
      if (std::scanf("%d %d", &P[r], &C[r]) != 2) return 2;
    mc_attn_params p{Hq, Hkv, D, 16, (int64_t)1 << 20, dtype, 0.f};
    int64_t n = -1;
    mc_status st = plan_items(&p, P.data(), C.data(), batch, kv_splits, nullptr, 0, &n);
    std::vector<int32_t> items((size_t)(n > 0 ? 4 * n : 4));
    if (st == MC_OK && n > 0) st = plan_items(&p, P.data(), C.data(), batch, kv_splits, items.data(), n, &n);
    int64_t total_new = 0;
    for (int32_t c : C) total_new += c > 0 ? c : 0;
    const size_t bytes = st == MC_OK ? list_bytes(&p, batch, total_new, kv_splits > 0 ? kv_splits : 1) : 0;
    std::printf("%d %lld %d %zu\n", (int)st, (long long)(st == MC_OK ? n : -1),
                (int)suggest_kv_splits(&p, P.data(), C.data(), batch), bytes);
    if (st == MC_OK)
      for (int64_t i = 0; i < n; ++i)
        std::printf("%d %d %d %d\n", items[4 * i], items[4 * i + 1], items[4 * i + 2], items[4 * i + 3]);
  }
}

int main(int argc, char** argv) {
  if (argc > 1 && std::string(argv[1]) == "plan") return run_plans();
  test_rejections();
  test_slot_ring();
  if (failures == 0) std::printf("selftest ok\n");
  return failures == 0 ? 0 : 1;
}
