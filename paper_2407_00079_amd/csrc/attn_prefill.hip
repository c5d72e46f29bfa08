// Prefix-reused, paged, chunked-prefill attention for gfx950 (paper Section 3,
// steps 1-2: the uncached tokens of a request attend to the reused prefix pages
// plus their own pages; the paper gives no kernel, this design is ours).
// This file: what both dtypes share in structure, the fp32 instantiation (32x32x2 MFMA tiles)
// and the merge of partial results.  The bf16 instantiation (16x16x32 MFMA tiles, two row
// tiles per wave) is attn_prefill_bf16.hip; it follows the same plan.
//
// Shape of the computation
//   * A workgroup owns a tile of stacked query rows of one (request, KV head):
//     row = token * G + head_in_group, so a K/V tile staged once in LDS feeds all
//     G query heads that share the KV head.  Each wave takes one block of 32 rows.
//   * Scores are computed TRANSPOSED, S^T = K Q^T, on MFMA tiles.  In the accumulator a
//     lane then owns query columns and a few keys per 32-key block, so the softmax row
//     reductions are in-lane plus an exchange between lane groups, and exp2(S^T) is
//     already laid out as the B operand of O^T += V^T P^T.  The key order inside that
//     contraction is the accumulator's row order; V^T fragments are fetched in the same
//     order (bf16: LDS transpose reads; f32: plain row reads).
//   * The KV loop walks the block table 64 keys (4 pages) at a time.  Tiles are
//     triple buffered in LDS and filled by direct global->LDS loads (no registers,
//     no LDS stores; one barrier per tile).  The 16-byte granules of a row are XOR
//     swizzled so that fragment reads are bank-conflict free; a fragment address is
//     (lane base XOR constant) + constant.  Tiles that lie wholly inside what every
//     row of the workgroup may see run a mask-free body; only tiles that touch the
//     chunk's diagonal compare key index against row position.
//   * Online softmax in fp32, base 2 (scale * log2 e folded into one fma).  Any
//     reference below overflow gives the same quotient O / l, so fully visible
//     blocks take no maxima at all: probabilities are formed against the reference
//     as it stands, and a block whose probabilities show that a score outgrew it
//     by more than 2^8 (fp32: by their sums; bf16: by a bit test on the rounded values)
//     is recomputed against its true maximum (rare; O is rescaled only then).  Blocks
//     on the chunk's diagonal take the masked, max-first path.
//   * Two waves per SIMD, half a step apart: while one wave's softmax occupies the
//     vector ALU under its score MFMAs, the other wave's P V MFMAs keep the matrix
//     pipe busy.  Waves of the second half whose rows lie past the chunk's end exit
//     at once (the barriers count surviving waves only).
#include <type_traits>

#include "attn_device.h"
#include "mc_internal.h"

namespace mc {
namespace {

// ---------------------------------------------------------------------------
// dtype traits: how fragments are fetched and multiplied
// ---------------------------------------------------------------------------
// bf16 rows as the merge kernel writes them (the bf16 attention kernel itself lives in attn_prefill_bf16.hip)
template <int D>
struct Bf16 {
  static constexpr int kD = D;
  static constexpr int kOutRowBytes = D * 2;
  // four consecutive output columns
  static __device__ __forceinline__ void store4(char* orow, int col, float a, float b, float c, float d) {
    bf16x4 v;
    v[0] = (__bf16)a;
    v[1] = (__bf16)b;
    v[2] = (__bf16)c;
    v[3] = (__bf16)d;
    *reinterpret_cast<bf16x4*>(orow + col * 2) = v;
  }
};

struct F32 {
  static constexpr int kD = 64;
  static constexpr int kOutRowBytes = kD * 4;
  static constexpr int kQKSteps = kD / 2;     // mfma 32x32x2 steps over head_dim
  static constexpr int kPVSteps = 16;         // one accumulator register (2 keys across halves) per step
  static constexpr int kDBlocks = kD / 32;
  typedef float frag;

  static __device__ __forceinline__ f32x16 mma(frag a, frag b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ frag load_q(const char* qrow, int kk, int half) {
    return *reinterpret_cast<const float*>(qrow + (kk * 2 + half) * 4);
  }
  static __device__ __forceinline__ int k_swz(int row) { return row & 15; }
  static __device__ __forceinline__ int v_swz(int) { return 0; }
  // column 2*kk + half lies in granule kk/2 at byte ((kk & 1) * 2 + half) * 4:
  // r*256 + ((kk/2) ^ (r & 15)) * 16 + ...  ==  (k_lane_off ^ ((kk/2) << 4)) + (kk & 1) * 8
  static __device__ __forceinline__ int k_lane_off(int lane) {
    const int r = lane & 31;
    return r * kRowBytes + ((r & 15) << 4) + (lane >> 5) * 4;
  }
  // A operand: K[32*kb + lane%32][2*kk + half]; kx[kk/2] = lane base ^ ((kk/2) << 4)
  static constexpr int kKX = kQKSteps / 2;
  static __device__ __forceinline__ uint32_t k_xor(int i) { return (uint32_t)(i << 4); }
  static __device__ __forceinline__ frag load_k(const uint32_t (&kx)[kKX], int off, int kk) {
    return *reinterpret_cast<MC_LDS const float*>(kx[kk >> 1] + (kk & 1) * 8 + off);
  }
  // step = accumulator register r: key 32*kb + 8*(r/4) + 4*half + r%4, column db*32 + lane%32
  static __device__ __forceinline__ int v_lane_off(int lane) { return (lane >> 5) * 4 * kRowBytes + (lane & 31) * 4; }
  static constexpr int kVX = 1;
  static __device__ __forceinline__ uint32_t v_xor(int) { return 0; }
  static __device__ __forceinline__ frag load_v(const uint32_t (&vx)[kVX], int off, int step, int db) {
    return *reinterpret_cast<MC_LDS const float*>(vx[0] + off + ((step >> 2) * 8 + (step & 3)) * kRowBytes + db * 128);
  }
  struct pblock { f32x16 p; };
  static __device__ __forceinline__ pblock round_p(const f32x16& p) { return pblock{p}; }
  static __device__ __forceinline__ frag p_frag(const pblock& b, int step) { return b.p[step]; }
  template <int N>
  static __device__ __forceinline__ float round_sum(pblock& b, const f32x16& p, int e0, float acc) {
    static_assert(N == 1, "f32 probabilities are taken one at a time");
    b.p[e0] = p[e0];
    return acc + p[e0];
  }
  static __device__ __forceinline__ float block_sum(const pblock& b) {
    float acc = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc += b.p[r];
    return acc;
  }
  static __device__ __forceinline__ void store4(char* orow, int col, float a, float b, float c, float d) {
    f32x4 v = {a, b, c, d};
    *reinterpret_cast<f32x4*>(orow + col * 4) = v;
  }
};

// ---------------------------------------------------------------------------
// kernel
// ---------------------------------------------------------------------------
// SPLIT: the work item covers only slice item.slice of the request's keys (whole 64-key tiles,
// ceil(tiles / kv_splits) per slice) and writes a PARTIAL result - the normalised fp32 output
// over its keys and their log-sum-exp (-inf where the slice holds no key the row may see) - for
// mc_attn_merge_lse to combine (paper Section 5.1: attention is associative over key slices).
template <class T, int WAVES, bool SPLIT>
__global__ __launch_bounds__(WAVES * 64) void attn_prefill_kernel(const AttnArgs a) {
  __shared__ __attribute__((aligned(16))) char smem[kBuffers * (kKTileBytes + kVTileBytes)];
  constexpr int kTileRows = WAVES * 32;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int half = lane >> 5;

  const AttnItem item = a.items[blockIdx.x];
  const AttnReq rq = a.reqs[item.req];
  const int G = a.G;
  const int P = rq.prefix;
  const int L = rq.prefix + rq.chunk;
  const int n_rows = rq.chunk * G;
  const int last_page = rq.pages - 1;

  // A wave of the second half (these copy no tiles) whose 32 rows all lie past the end of the chunk
  // has nothing to do: it ends here, and the workgroup's barriers then wait for the surviving
  // waves only.  Small chunks (a 16-token chunk of an 8-head group fills 4 of 8 waves) then
  // spend no MFMA work on rows that are never stored.
  if (wave >= WAVES / 2 && item.row0 + wave * 32 >= n_rows) return;

  // ---- this lane's query row: its Q fragments stay in registers for the whole KV loop
  typename T::frag qf[T::kQKSteps];
  int row = item.row0 + wave * 32 + (lane & 31);
  const bool live = row < n_rows;
  row = live ? row : n_rows - 1;                // dead rows recompute the last row, never stored
  const int tok = row / G;                      // token index inside the chunk
  const int qhead = item.kv_head * G + (row - tok * G);
  {
    const char* qrow = reinterpret_cast<const char*>(a.q) + ((int64_t)(rq.q_off + tok) * a.Hq + qhead) * kRowBytes;
#pragma unroll
    for (int kk = 0; kk < T::kQKSteps; ++kk) qf[kk] = T::load_q(qrow, kk, half);
  }

  // ---- keys this workgroup needs, and how many leading tiles need no mask
  const int tok_first = item.row0 / G;
  int tok_last = (item.row0 + kTileRows - 1) / G;
  tok_last = tok_last < rq.chunk - 1 ? tok_last : rq.chunk - 1;
  const int kv_end = P + tok_last + 1;                       // <= L
  int n_tiles = (kv_end + kTileKeys - 1) / kTileKeys;        // tiles [t_lo, n_tiles) are this item's
  int t_lo = 0;
  if (SPLIT) {
    const int per = ((L + kTileKeys - 1) / kTileKeys + a.kv_splits - 1) / a.kv_splits;
    t_lo = item.slice * per;
    n_tiles = n_tiles < t_lo + per ? n_tiles : t_lo + per;
  }
  int n_free = (P + tok_first + 1) / kTileKeys;              // every key of these tiles is visible to every row
  n_free = n_free < n_tiles ? n_free : n_tiles;
  // where this lane's row goes: the output itself, or this slice's plane of the partials
  const int64_t orow_idx = (int64_t)(rq.q_off + tok) * a.Hq + qhead;
  if (SPLIT && t_lo >= n_tiles) {
    // no key of the slice is visible to any row of the tile
    if (live) {
      char* orow = reinterpret_cast<char*>(a.o_parts) + ((int64_t)item.slice * a.rows_total + orow_idx) * (T::kD * 4);
#pragma unroll
      for (int db = 0; db < T::kDBlocks; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
          *reinterpret_cast<f32x4*>(orow + (db * 32 + q4 * 8 + half * 4) * 4) = f32x4{0.f, 0.f, 0.f, 0.f};
      if (half == 0) a.lse_parts[(int64_t)item.slice * a.rows_total + orow_idx] = -INFINITY;
    }
    return;
  }

  // ---- global -> LDS, no registers in between.  One wave instruction writes 1 KiB of LDS (lane i
  //      its 16 bytes at +16*i): 4 tile rows x 16 granules, all inside one page.  Lane i fetches,
  //      for LDS granule position i%16 of row i/16, the logical granule (i%16) ^ swz(row).
  //      Only the first half of the waves issue copies: they are the first wave of each SIMD, win
  //      the issue arbitration against the second wave and would otherwise idle at the tile
  //      barrier, and a copy instruction holds its wave for ~130 cycles.  Fetching wave w copies
  //      chunks w, w + kFetchWaves, ... of the tile (chunk c = rows 4c..4c+3, page c/4).
  constexpr int kFetchWaves = WAVES / 2;
  constexpr int kChunks = kTileKeys / 4;                      // 1 KiB chunks per K (or V) tile
  constexpr int kFetch = kChunks / kFetchWaves;               // chunks per fetching wave
  static_assert(kChunks % kFetchWaves == 0 && kFetch <= 8, "tile must split evenly over the fetching waves");
  const char* kbase = reinterpret_cast<const char*>(a.k_pool) + (int64_t)item.kv_head * kPageHeadBytes;
  const char* vbase = reinterpret_cast<const char*>(a.v_pool) + (int64_t)item.kv_head * kPageHeadBytes;
  const int64_t page_stride = (int64_t)a.Hkv * kPageHeadBytes;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const uint32_t smem_base = (uint32_t)(uintptr_t)(MC_LDS char*)smem;
  const bool fetcher = wave_u < kFetchWaves;
  // The block table is read through the scalar cache (it is constant while the kernel runs),
  // one tile AHEAD of the K/V loads that need it, so no wave ever waits for a page id.
  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  const_i32_ptr btc = (const_i32_ptr)(a.block_tables + (int64_t)item.req * a.max_pages);
  const int64_t first_page_off = (int64_t)btc[0] * page_stride;   // page of key 0: always valid
  int pid[kFetch];

  int pid_next[kFetch];
  // ids of tile `tile` into pid_next (issued before a barrier, so the scalar loads complete under it)
  auto load_ids = [&](int tile) __attribute__((always_inline)) {
    if (!fetcher) return;
#pragma unroll
    for (int i = 0; i < kFetch; ++i) {
      int lp = tile * (kTileKeys / kPageTokens) + (wave_u + i * kFetchWaves) / 4;
      lp = lp < last_page ? lp : last_page;                  // never index the table past the request's pages
      pid_next[i] = btc[lp];
    }
  };
  auto take_ids = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < kFetch; ++i) pid[i] = pid_next[i];
  };
  // Per-lane byte offset inside a (page, head) block: the same for every chunk of a wave, because
  // a wave's chunks are 16 rows (one page) apart and both swizzles depend on row % 16 only.
  const int lane_row = (wave_u & 3) * 4 + (lane >> 4);       // row of the page this lane copies a granule of
  const uint32_t k_src = (uint32_t)(lane_row * kRowBytes + (((lane & 15) ^ T::k_swz(lane_row)) << 4));
  const uint32_t v_src = (uint32_t)(lane_row * kRowBytes + (((lane & 15) ^ T::v_swz(lane_row)) << 4));
  static_assert(kFetchWaves % 4 == 0, "a fetching wave's chunks must all sit at the same rows of their pages");
  // enqueue the copy of tile `tile` (page ids in pid[]) into LDS buffer `buf`
  auto fetch = [&](int tile, int buf) __attribute__((always_inline)) {
    if (!fetcher) return;
    const uint32_t dst0 = smem_base + buf * kKTileBytes + wave_u * 1024;
    if ((tile + 1) * kTileKeys <= L) {
      // whole tile inside the sequence: scalar page base + constant lane offset
#pragma unroll
      for (int i = 0; i < kFetch; ++i) {
        const int64_t page_off = (int64_t)pid[i] * page_stride;
        const uint32_t dst = dst0 + i * kFetchWaves * 1024;
        dma16(kbase + page_off, k_src, dst);
        dma16(vbase + page_off, v_src, dst + kVBase);
      }
    } else {
      // Slots at or past the request's length may hold anything (NaN would survive p = 0 in P V):
      // those lanes copy row 0 of the request's first page instead; the causal mask hides the key.
#pragma unroll
      for (int i = 0; i < kFetch; ++i) {
        const int row = (wave_u + i * kFetchWaves) * 4 + (lane >> 4);
        const bool in_seq = tile * kTileKeys + row < L;
        const int64_t page_off = (int64_t)pid[i] * page_stride;
        const char* ks = kbase + (in_seq ? page_off + k_src : first_page_off + (k_src & 255));
        const char* vs = vbase + (in_seq ? page_off + v_src : first_page_off + (v_src & 255));
        const uint32_t dst = dst0 + i * kFetchWaves * 1024;
        dma16(ks, dst);
        dma16(vs, dst + kVBase);
      }
    }
  };
  // wait until this wave's copies have landed (vmcnt(0); the other counters are left alone)
  auto copies_landed = [&]() __attribute__((always_inline)) { __builtin_amdgcn_s_waitcnt(0x0F70); };

  // ---- running softmax state and output accumulators (O^T: registers index head_dim)
  f32x16 o[T::kDBlocks];
  float m_run = -INFINITY;   // reference of the probabilities accumulated so far (log2 units)
  float l_sum = 0.f;         // this lane's share of the row sum (halves merged at the end)
#pragma unroll
  for (int db = 0; db < T::kDBlocks; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  const float c = a.scale_log2e;
  const uint32_t k_lane = smem_base + T::k_lane_off(lane);
  const uint32_t v_lane = smem_base + kVBase + T::v_lane_off(lane);
  // lane bases with the swizzle's XOR already applied: a fragment address is one of these plus a
  // constant, and in the pipeline (buffer known at compile time) that constant is an immediate
  uint32_t kx[T::kKX], vx[T::kVX];
#pragma unroll
  for (int i = 0; i < T::kKX; ++i) kx[i] = k_lane ^ T::k_xor(i);
#pragma unroll
  for (int i = 0; i < T::kVX; ++i) vx[i] = v_lane ^ T::v_xor(i);

  // ---- building blocks that are NOT on the steady-state path (prologue, last block, rare recompute)
  // S^T block = K Q^T for keys [32*kb, 32*kb+32) of the tile in LDS buffer `buf`, one K fragment
  // in flight at a time (it runs where registers are scarce)
  auto qk_block = [&](int buf, int kb, f32x16& s) __attribute__((always_inline)) {
    const int off = buf * kKTileBytes + kb * 32 * kRowBytes;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < T::kQKSteps; ++kk) {
      const typename T::frag kf = T::load_k(kx, off, kk);
      s = T::mma(kf, qf[kk], s);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // Mask a block if it reaches the diagonal, take the TRUE column maxima and raise the reference
  // m_run if some column outgrew it by more than the slack (rare, wave-uniform branch; always taken
  // for the first block, m_run starts at -inf).
  auto settle_reference = [&](f32x16& s, int key0, auto masked_tag) __attribute__((always_inline)) {
    constexpr bool kMasked = decltype(masked_tag)::value;
    if (kMasked) {
      // key of register r: key0 + 8*(r/4) + 4*half + r%4; visible iff <= P + tok
      const int lim = P + tok - key0 - half * 4;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = ((r >> 2) * 8 + (r & 3) <= lim) ? s[r] : -INFINITY;
    }
    float mx = s[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
    mx = max_with_other_half(mx) * c;
    if (__builtin_amdgcn_ballot_w64(mx > m_run + kRescaleSlack) != 0) {
      const float m_new = fmaxf(m_run, mx);
      // a row that has seen no key yet keeps m_run = -inf (possible only in a slice that starts
      // beyond the row's diagonal): nothing to rescale, and -inf - -inf must not reach exp2
      const float alpha = (SPLIT && m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);
      l_sum *= alpha;
      m_run = m_new;
#pragma unroll
      for (int db = 0; db < T::kDBlocks; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
    }
  };
  // scores -> probabilities against the reference as it stands, rounded the way P V multiplies them;
  // returns this lane's share of the block's column sums
  auto probabilities = [&](const f32x16& s, typename T::pblock& pb) __attribute__((always_inline)) {
    f32x16 p;
    const float m_ref = SPLIT ? fmaxf(m_run, kNoKeyYet) : m_run;
#pragma unroll
    for (int r = 0; r < 16; ++r) p[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -m_ref));
    pb = T::round_p(p);
    return T::block_sum(pb);
  };
  // O^T += V^T P^T for the block's 32 keys, V fragments read just in time
  auto pv_block = [&](int buf, int kb, const typename T::pblock& pb) __attribute__((always_inline)) {
    const int off = buf * kVTileBytes + kb * 32 * kRowBytes;
#pragma unroll
    for (int st = 0; st < T::kPVSteps; ++st)
#pragma unroll
      for (int db = 0; db < T::kDBlocks; ++db) o[db] = T::mma(T::load_v(vx, off, st, db), T::p_frag(pb, st), o[db]);
  };

  // ---- KV loop.  Software pipeline over 32-key blocks, scheduled by hand: the order written
  //      below is the order issued (a scheduling barrier closes every group).
  //
  //      One step has two phases and one ring of kRing fragment registers:
  //        phase A  scores of block j+1: MFMA i multiplies ring[i] (K fragment i of block j+1, read
  //                 during the previous phase B) and frees it; the V fragment that P V step i of
  //                 block j needs is read into the freed slot; under these MFMAs the vector ALU
  //                 turns the scores of block j into probabilities, a group's share per MFMA.
  //        phase B  P V of block j: MFMA i multiplies ring[i] (the V fragment) and frees it; K
  //                 fragment i of block j+2 is read into the freed slot.
  //      Every LDS read is thus issued about a phase (8 MFMAs) before its consumer.
  //      Tiles are triple buffered in LDS: the copy of tile t+2 is enqueued at the start of
  //      tile t (right after the one barrier per tile), into the buffer tile t-1 has just left.
  constexpr int kRing = T::kQKSteps;
  static_assert(kRing == T::kPVSteps * T::kDBlocks, "both phases must have the same number of MFMAs");
  constexpr int kPer = kRing >= 16 ? 1 : 16 / kRing;      // scores turned into probabilities per active group
  constexpr int kEvery = kRing >= 16 ? kRing / 16 : 1;    // every kEvery-th group is active
  typename T::frag ring[kRing];
  f32x16 s_cur, s_next;
  auto load_k_ring = [&](int buf, int kb) __attribute__((always_inline)) {
    const int off = buf * kKTileBytes + kb * 32 * kRowBytes;
#pragma unroll
    for (int i = 0; i < kRing; ++i) ring[i] = T::load_k(kx, off, i);
  };

  // The pipeline only ever sees fully visible blocks, and it takes no maxima.  Probabilities are formed
  // against the reference as it stands and the block sums tell whether that was safe: a lane's sum
  // of 16 probabilities above kSumGuard (or not finite) means some score outgrew the reference by
  // more than the slack.  Only then (rare, wave-uniform) the block's scores are recomputed from
  // the tile still in LDS, the reference is raised to their true maximum and the probabilities
  // are redone; nothing has been accumulated from the discarded ones.
  constexpr float kSumGuard = 4096.0f;   // 16 probabilities of at most 2^kRescaleSlack each
  // block j = (buf_cur, kb_cur); block j+2 = (buf_pre, kb_pre)
  typename T::pblock pb;
  auto phase_a = [&](int buf_cur, int kb_cur) __attribute__((always_inline)) {
    const int off_v = buf_cur * kVTileBytes + kb_cur * 32 * kRowBytes;
    s_cur = s_next;
#pragma unroll
    for (int r = 0; r < 16; ++r) s_next[r] = 0.f;
    float bsum = 0.f;
    const float m_ref = SPLIT ? fmaxf(m_run, kNoKeyYet) : m_run;
#pragma unroll
    for (int i = 0; i < kRing; ++i) {
      s_next = T::mma(ring[i], qf[i], s_next);
      ring[i] = T::load_v(vx, off_v, i / T::kDBlocks, i % T::kDBlocks);
      if (i % kEvery == 0) {
        const int e0 = i / kEvery * kPer;
#pragma unroll
        for (int e = e0; e < e0 + kPer; ++e) s_cur[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[e], c, -m_ref));
        // rounding and summing trail one group behind the exponentials they depend on
        if (i > 0) bsum = T::template round_sum<kPer>(pb, s_cur, e0 - kPer, bsum);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    bsum = T::template round_sum<kPer>(pb, s_cur, 16 - kPer, bsum);
    if (__builtin_amdgcn_ballot_w64(!(bsum <= kSumGuard)) != 0) {
      qk_block(buf_cur, kb_cur, s_cur);
      settle_reference(s_cur, 0, std::false_type{});
      bsum = probabilities(s_cur, pb);
    }
    l_sum += bsum;
  };
  auto phase_b = [&](int buf_pre, int kb_pre) __attribute__((always_inline)) {
    const int off_k = buf_pre * kKTileBytes + kb_pre * 32 * kRowBytes;
#pragma unroll
    for (int i = 0; i < kRing; ++i) {
      o[i % T::kDBlocks] = T::mma(ring[i], T::p_frag(pb, i / T::kDBlocks), o[i % T::kDBlocks]);
      ring[i] = T::load_k(kx, off_k, i);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // One block start to finish, for the few blocks that may reach the diagonal: scores (unless the
  // pipeline has left them in `s`), mask, true maxima and reference, probabilities, P V.
  auto plain_block = [&](int buf, int kb, int key0, f32x16& s, bool have_scores) __attribute__((always_inline)) {
    if (!have_scores) qk_block(buf, kb, s);
    settle_reference(s, key0, std::true_type{});
    typename T::pblock pb;
    l_sum += probabilities(s, pb);
    pv_block(buf, kb, pb);
  };

  load_ids(t_lo);
  take_ids();
  fetch(t_lo, 0);
  load_ids(t_lo + 1);
  take_ids();
  if (n_tiles > t_lo + 1) {
    fetch(t_lo + 1, 1);
    load_ids(t_lo + 2);
    take_ids();
  }
  // everything issued so far has landed (Q fragments, tiles 0 and 1): inside the loop the
  // vector-memory counter only ever counts the tile copies
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  int buf = 0;
  // One tile = barrier, enqueue the copy of tile + 2, two blocks.  After the barrier tile + 1 is
  // visible to every wave (it was enqueued a whole tile ago) and no wave reads tile - 1 any
  // more, so that buffer takes tile + 2.
  auto tile_sync = [&](int tile) __attribute__((always_inline)) {
    const bool ahead = tile + 2 < n_tiles;
    if (ahead) load_ids(tile + 3);
    copies_landed();
    __syncthreads();
    if (ahead) {
      fetch(tile + 2, buf == 0 ? 2 : buf - 1);   // (tile + 2) % 3, ids loaded one tile ago
      take_ids();
    }
  };
  int tile = t_lo;
  // tiles every key of which is visible to every row go through the pipeline (never the last
  // tile: the pipeline always computes the scores of one block ahead)
  const int n_plain = n_free < n_tiles - 1 ? n_free : n_tiles - 1;
  qk_block(0, 0, s_next);
  if (tile < n_plain) {
    settle_reference(s_next, 0, std::false_type{});
    load_k_ring(0, 1);
    // The two waves of a SIMD run half a step apart: the second one (waves WAVES/2 ..) passes the
    // tile barrier between the two phases of the tile's first step instead of before it.  When
    // the barrier opens one wave of each SIMD starts a phase A (a dependent MFMA chain under
    // heavy vector work) and the other a phase B (independent MFMAs, no vector work), so the
    // matrix pipe always has an MFMA that is ready and the vector ALU is never wanted twice.
    // Safe because phase A of a tile's first step reads nothing of the tile before it and
    // nothing of the tile after it, and every wave still passes one barrier per tile.
    const bool late_barrier = wave_u >= WAVES / 2;
    // The loop body is written out for the three buffers in turn, so that inside it every tile
    // offset is a compile-time constant and goes into the LDS instructions' immediate fields.
    auto pipelined_tile = [&](auto buf_tag) __attribute__((always_inline)) {
      constexpr int b = decltype(buf_tag)::value, bn = (b + 1) % kBuffers;
      buf = b;
      if (!late_barrier) tile_sync(tile);
      phase_a(b, 0);               // block 0: scores of block 1 ...
      if (late_barrier) tile_sync(tile);
      phase_b(bn, 0);              // ... then the K fragments of the next tile's block 0
      phase_a(b, 1);               // block 1: scores of the next tile's block 0 ...
      phase_b(bn, 1);              // ... then the K fragments of its block 1
      buf = bn;
      ++tile;
    };
    for (;;) {
      if (tile >= n_plain) break;
      pipelined_tile(std::integral_constant<int, 0>{});
      if (tile >= n_plain) break;
      pipelined_tile(std::integral_constant<int, 1>{});
      if (tile >= n_plain) break;
      pipelined_tile(std::integral_constant<int, 2>{});
    }
  }
  // the rest may reach the diagonal: block at a time; the scores of the first such block are in s_next
  bool have_scores = true;
  for (; tile < n_tiles; ++tile) {
    const int buf_next = buf == 2 ? 0 : buf + 1;
    tile_sync(tile);
    plain_block(buf, 0, tile * kTileKeys, s_next, have_scores);
    have_scores = false;
    plain_block(buf, 1, tile * kTileKeys + 32, s_next, false);
    buf = buf_next;
  }
  const float l_run = sum_with_other_half(l_sum);

  // ---- epilogue: normalise, round, store; lane holds 4 consecutive columns per (db, r/4)
  if (live && !SPLIT) {
    const float inv = 1.0f / l_run;
    char* orow = reinterpret_cast<char*>(a.out) + orow_idx * kRowBytes;
#pragma unroll
    for (int db = 0; db < T::kDBlocks; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int col = db * 32 + q4 * 8 + half * 4;
        T::store4(orow, col, o[db][q4 * 4 + 0] * inv, o[db][q4 * 4 + 1] * inv, o[db][q4 * 4 + 2] * inv,
                  o[db][q4 * 4 + 3] * inv);
      }
    if (a.lse != nullptr && half == 0) a.lse[orow_idx] = (m_run + __builtin_amdgcn_logf(l_run)) * 0.6931471805599453f;
  }
  if (live && SPLIT) {
    // partial result in fp32; a row that saw no key of the slice has l = 0: zeros and -inf
    const float inv = l_run > 0.f ? 1.0f / l_run : 0.f;
    char* orow = reinterpret_cast<char*>(a.o_parts) + ((int64_t)item.slice * a.rows_total + orow_idx) * (T::kD * 4);
#pragma unroll
    for (int db = 0; db < T::kDBlocks; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
        *reinterpret_cast<f32x4*>(orow + (db * 32 + q4 * 8 + half * 4) * 4) =
            f32x4{o[db][q4 * 4 + 0] * inv, o[db][q4 * 4 + 1] * inv, o[db][q4 * 4 + 2] * inv, o[db][q4 * 4 + 3] * inv};
    if (half == 0)
      a.lse_parts[(int64_t)item.slice * a.rows_total + orow_idx] =
          l_run > 0.f ? (m_run + __builtin_amdgcn_logf(l_run)) * 0.6931471805599453f : -INFINITY;
  }
}

// ---------------------------------------------------------------------------
// merge of partial results (paper Section 5.1: attention is associative over key slices):
//   lse = log sum_s exp(lse_s),  out = sum_s exp(lse_s - lse) o_s
// A thread owns 4 consecutive columns of one row and every SL-th part, starting at its split
// lane; a part whose lse is -inf has weight 0 and is not read.  D / 4 * SL threads per row, rows
// packed into 256-thread workgroups.  SL = 1 walks all parts in one thread (many rows, few
// parts); SL = 8 shortens the chain of dependent loads eightfold and adds the lanes' partial
// sums through LDS (few rows, many parts: small chunks against long prefixes).
// ---------------------------------------------------------------------------
template <typename T, int SL>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float* __restrict__ o_parts,
                                                         const float* __restrict__ lse_parts, int kv_splits,
                                                         int64_t rows, void* __restrict__ out,
                                                         float* __restrict__ lse) {
  constexpr int kThreadsPerRow = T::kD / 4;
  constexpr int kRows = 256 / (kThreadsPerRow * SL);     // rows of one workgroup
  __shared__ float red[kRows][SL];
  __shared__ f32x4 part[kRows][SL][kThreadsPerRow];
  const int rl = threadIdx.x / (kThreadsPerRow * SL);
  const int sl = (threadIdx.x / kThreadsPerRow) % SL;
  const int cl = threadIdx.x % kThreadsPerRow;
  const int col = cl * 4;
  const int64_t row_raw = (int64_t)blockIdx.x * kRows + rl;
  const bool live = row_raw < rows;
  const int64_t row = live ? row_raw : rows - 1;         // rows past the end compute the last row again and store nothing
  float m = -INFINITY;
  for (int s = sl; s < kv_splits; s += SL) m = fmaxf(m, lse_parts[(int64_t)s * rows + row]);
  if constexpr (SL > 1) {
    if (cl == 0) red[rl][sl] = m;
    __syncthreads();
#pragma unroll
    for (int t = 0; t < SL; ++t) m = fmaxf(m, red[rl][t]);
    __syncthreads();
  }
  float z = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if (m != -INFINITY) {
    for (int s = sl; s < kv_splits; s += SL) {
      const float w = __expf(lse_parts[(int64_t)s * rows + row] - m);
      if (w == 0.f) continue;
      z += w;
      const f32x4 v = *reinterpret_cast<const f32x4*>(o_parts + ((int64_t)s * rows + row) * T::kD + col);
      acc += w * v;
    }
  }
  if constexpr (SL > 1) {
    if (cl == 0) red[rl][sl] = z;
    part[rl][sl][cl] = acc;
    __syncthreads();
    if (sl != 0) return;
    z = 0.f;
    acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < SL; ++t) {
      z += red[rl][t];
      acc += part[rl][t][cl];
    }
  }
  if (!live) return;
  if (m != -INFINITY) acc *= 1.0f / z;
  T::store4(reinterpret_cast<char*>(out) + row * T::kOutRowBytes, col, acc[0], acc[1], acc[2], acc[3]);
  if (lse != nullptr && col == 0) lse[row] = m != -INFINITY ? m + __logf(z) : -INFINITY;
}

}  // namespace

hipError_t launch_attn(int dtype, const AttnArgs& args, hipStream_t stream) {
  (void)hipGetLastError();   // drop any stale error of earlier, unrelated runtime calls
  const bool split = args.kv_splits > 0;
  if (dtype == MC_DTYPE_BF16) return launch_attn_bf16(args, stream);
  if (split) attn_prefill_kernel<F32, kWaves, true><<<args.n_items, kWaves * 64, 0, stream>>>(args);
  else attn_prefill_kernel<F32, kWaves, false><<<args.n_items, kWaves * 64, 0, stream>>>(args);
  return hipGetLastError();
}

template <typename T, int SL>
static void enqueue_merge(const float* o_parts, const float* lse_parts, int kv_splits, int64_t rows, void* out,
                          float* lse, hipStream_t stream) {
  const int64_t per = 256 / (T::kD / 4 * SL);
  attn_merge_kernel<T, SL><<<(unsigned)((rows + per - 1) / per), 256, 0, stream>>>(o_parts, lse_parts, kv_splits,
                                                                                   rows, out, lse);
}

hipError_t launch_attn_merge(int dtype, int head_dim, const float* o_parts, const float* lse_parts, int kv_splits,
                             int64_t rows, void* out, float* lse, hipStream_t stream) {
  (void)hipGetLastError();
  const bool wide = kv_splits >= 8;   // enough parts to give each of 8 split lanes one
  if (dtype == MC_DTYPE_BF16 && head_dim == 128) {
    if (wide) enqueue_merge<Bf16<128>, 8>(o_parts, lse_parts, kv_splits, rows, out, lse, stream);
    else enqueue_merge<Bf16<128>, 1>(o_parts, lse_parts, kv_splits, rows, out, lse, stream);
  } else if (dtype == MC_DTYPE_BF16 && head_dim == 64) {
    if (wide) enqueue_merge<Bf16<64>, 8>(o_parts, lse_parts, kv_splits, rows, out, lse, stream);
    else enqueue_merge<Bf16<64>, 1>(o_parts, lse_parts, kv_splits, rows, out, lse, stream);
  } else if (dtype == MC_DTYPE_F32 && head_dim == 64) {
    if (wide) enqueue_merge<F32, 8>(o_parts, lse_parts, kv_splits, rows, out, lse, stream);
    else enqueue_merge<F32, 1>(o_parts, lse_parts, kv_splits, rows, out, lse, stream);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace mc
