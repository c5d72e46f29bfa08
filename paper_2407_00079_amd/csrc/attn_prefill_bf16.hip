// bf16 instantiation of the prefix-reused, paged, chunked-prefill attention (paper Section 3,
// steps 1-2; the kernel design is ours) on 16x16x32 MFMA tiles.
//
// Why this tile shape.  The board holds its power limit by lowering the shader clock, and the
// energy of a bf16 MFMA per flop depends on its shape: a loop of v_mfma_f32_16x16x32_bf16 runs
// at ~2.0 GHz where the same flops as v_mfma_f32_32x32x16_bf16 run at ~1.75 GHz (a 16x16x32
// tile reads and writes a quarter of the accumulator registers per instruction and half per
// flop).  What a 16x16 tile would cost elsewhere - twice the operand fragments per flop - is
// avoided by giving every wave TWO row tiles: each K or V fragment read from LDS feeds two
// MFMAs, so the LDS traffic per flop is that of the 32x32 form.
//
// Shape of the computation (see attn_prefill.hip for what is common to both dtypes)
//   * A wave owns 32 stacked query rows as two row tiles of 16; lane l serves rows l % 16 of
//     both tiles and, of every 32-key block, the 8 keys 4 (l / 16) + {0..3} and 16 + 4 (l / 16)
//     + {0..3} - the rows of its lane group in the two 16x16 score tiles S^T = K Q^T.  The
//     probabilities of a lane are therefore already the B operand of O^T += V^T P^T (a 32-key
//     contraction in that key order); V^T fragments are fetched in the same order with two LDS
//     transpose reads.  Row maxima (diagonal tiles and the rare recompute path only) are in-lane
//     over 8 values plus an exchange between the 4 lane groups.
//   * Per 32-key block at head_dim 128: 16 score MFMAs (2 key tiles x 2 row tiles x 4 head_dim
//     steps of 32) and 16 P V MFMAs (8 head_dim tiles x 2 row tiles), 8 K fragments and 8 V
//     fragments from LDS; at head_dim 64 half of each (see Geo).
//   * K/V tiles, their copy into LDS, the page walk, the lazy softmax reference, the two-phase
//     ring schedule and the half-step skew of the two waves of a SIMD are those of
//     attn_prefill.hip; the swizzles differ (fragment shapes differ).
//   * Vector instructions are what the matrix pipe does not hide here (each one costs its issue
//     time, measured by removing them one kind at a time), so the softmax keeps only what it
//     cannot do without: per score one fma and one exp2, per pair one rounding to bf16.  The row
//     sums of the rounded probabilities come from two more MFMAs per block (ones x P^T), and the
//     guard of the lazy reference is an OR over the packed probabilities (see kRefLift).
#include <type_traits>

#include "attn_device.h"
#include "mc_internal.h"

namespace mc {
namespace {

typedef bf16x8 frag;
typedef f32x4 acc4;

// The reference of a row's probabilities is kept kRefLift (log2 units) ABOVE the largest score it was last set
// from, so probabilities are at most 2^-7 then and stay below 2 while later scores outgrow that maximum by less
// than 8: "some probability reached 2" is bit 14 of a bf16 pattern, which an OR over the block's packed
// probabilities finds (bit 14 is also set in inf and NaN).  The reference is raised when a score comes within
// kRaiseAbove of making its probability 2, which is before the guard can fire.
constexpr float kRefLift = 7.0f;
constexpr float kRaiseAbove = 0.5f;
constexpr uint32_t kGuardBits = 0x40004000u;

__device__ __forceinline__ acc4 mma(frag a, frag b, acc4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// Tile geometry for head_dim D (128: 256-byte rows, 64: 128-byte rows).
template <int D>
struct Geo {
  static_assert(D == 128 || D == 64, "head_dim");
  static constexpr int kRowB = D * 2;                    // bytes of a Q, K, V or O row
  static constexpr int kGran = kRowB / 16;               // 16-byte granules of a row
  static constexpr int kLineShift = D == 128 ? 0 : 1;    // log2 of the rows that share a 256-byte line of LDS banks
  static constexpr int kSteps = D / 32;                  // contraction steps of the scores over head_dim
  static constexpr int kDTiles = D / 16;                 // 16-column tiles of the output
  static constexpr int kRing = kDTiles;                  // K fragments of a block = V fragments of a block
  static_assert(kRing == 2 * kSteps, "both phases walk the ring once");
  static constexpr int kPageHeadB = kPageTokens * kRowB; // one (page, KV head), contiguous in the pool
  static constexpr int kKTileB = kTileKeys * kRowB;      // a K (or V) tile in LDS; rows dense, granules swizzled
  static constexpr int kVBaseB = kBuffers * kKTileB;     // the K tiles of the three buffers, then the V tiles
  static constexpr int kChunkRows = 1024 / kRowB;        // rows one wave copy instruction (1 KiB) covers
  static constexpr int kPageChunks = kPageTokens / kChunkRows;

  // LDS swizzles: 16-byte granule g of tile row r is stored at granule g ^ swz(r).  The banks repeat every
  // 256 bytes, i.e. every row (D 128) or every second row (D 64).
  // K: a fragment read has 16 lanes on 16 consecutive rows at the same logical granule -> spread them over
  //    all 16 granule positions of a 256-byte line (D 64: two rows per line, 8 positions each).
  // V: a transpose read has 32 lanes on 8 consecutive rows x 32 bytes -> the 32-byte piece of a row moves
  //    with the line number, so the 8 rows cover all banks.
  static __device__ __forceinline__ int k_swz(int row) { return (row >> kLineShift) & (kGran - 1); }
  static __device__ __forceinline__ int v_swz(int row) { return ((row >> kLineShift) & (kGran / 2 - 1)) << 1; }

  // K fragment (key tile kt, head_dim step c) of a block: lane (j = l % 16, g = l / 16) reads
  // K[16 kt + j][32 c + 8 g .. + 7], i.e. granule 4 c + g of row 16 kt + j, stored at (4 c) ^ g ^ swz(j)
  // (the swizzle of row 16 kt + j is that of row j):  address = k_lane_off ^ (c << 6)  (+ row offset)
  static __device__ __forceinline__ int k_lane_off(int lane) {
    const int j = lane & 15, g = lane >> 4;
    return j * kRowB + ((g ^ k_swz(j)) << 4);
  }
  // ring slot i of a block's scores = (step i / 2, key tile i % 2)
  static __device__ __forceinline__ frag load_k(const uint32_t (&kx)[kSteps], int off, int i) {
    return *reinterpret_cast<MC_LDS const frag*>(kx[i >> 1] + off + (i & 1) * 16 * kRowB);
  }
  // V^T fragment (head_dim tile dt) of a block: lane (j, g) needs V[key][16 dt + j] for the keys 4 g + {0..3}
  // and 16 + 4 g + {0..3}.  The transpose read returns, to lane i of a 16-lane group, element i % 4 of
  // lanes i / 4, 4 + i / 4, 8 + i / 4, 12 + i / 4: source lane s addresses key 4 g + s / 4, columns
  // 16 dt + 4 (s % 4) .. + 3.  That is 8 bytes at byte 32 dt + 8 (s % 4) of row rr = 4 g + s / 4: 32-byte piece
  // dt, stored at piece dt ^ (v_swz(rr) / 2) (rows rr and rr + 16 swizzle alike):  address = v_lane_off ^ (dt << 5)
  static __device__ __forceinline__ int v_lane_off(int lane) {
    const int s = lane & 15, g = lane >> 4;
    const int rr = 4 * g + (s >> 2);
    return rr * kRowB + (v_swz(rr) << 4) + (((s & 3) >> 1) << 4) + ((s & 1) << 3);
  }
  static __device__ __forceinline__ frag load_v(const uint32_t (&vx)[kDTiles], int off, int dt) {
    const uint32_t p = vx[dt] + off;
    bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((MC_LDS bf16x4*)(uintptr_t)(p));
    bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((MC_LDS bf16x4*)(uintptr_t)(p + 16 * kRowB));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  }
};

// largest of a value over the 4 lane groups that share a query row (lanes l, l ^ 16, l ^ 32, l ^ 48)
__device__ __forceinline__ float max_over_groups(float x) {
  x = fmaxf(x, __shfl_xor(x, 16, 64));
  return max_with_other_half(x);
}

// The scores of one 32-key block as a lane holds them: s[rt][kt] is the accumulator of score tile
// (key tile kt, row tile rt); its register r is key 16 kt + 4 g + r of the block, row 16 rt + j.
struct Scores {
  acc4 t[2][2];
  // e = 8 rt + 4 kt + r
  __device__ __forceinline__ float get(int e) const { return t[e >> 3][(e >> 2) & 1][e & 3]; }
  __device__ __forceinline__ void set(int e, float v) { t[e >> 3][(e >> 2) & 1][e & 3] = v; }
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) t[rt][kt] = acc4{0.f, 0.f, 0.f, 0.f};
  }
};
// a block's probabilities as P V multiplies them: per row tile, the B operand of the 32-key step, kept as four
// words of two bf16 each (word k = keys 2 k, 2 k + 1 of the lane's eight)
struct PBlock {
  u32x4 w[2];
  __device__ __forceinline__ frag f(int rt) const { return __builtin_bit_cast(frag, w[rt]); }
};
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;

// round probabilities e, e + 1 (same row tile) into their fragment
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void round_pair(PBlock& b, const Scores& p, int e) {
  const f32x2 pp = {p.get(e), p.get(e + 1)};
  const bf16x2 pr = __builtin_convertvector(pp, bf16x2);      // one v_cvt_pk_bf16_f32 (round to nearest even)
  b.w[e >> 3][(e & 7) >> 1] = __builtin_bit_cast(uint32_t, pr);
}
template <int D, int WAVES, bool SPLIT>
__global__ __launch_bounds__(WAVES * 64) void attn_prefill_bf16_kernel(const AttnArgs a) {
  typedef Geo<D> X;
  // (these names hide the 256-byte-row constants of attn_device.h inside this kernel)
  constexpr int kD = D, kSteps = X::kSteps, kDTiles = X::kDTiles, kRing = X::kRing, kRowBytes = X::kRowB,
                kPageHeadBytes = X::kPageHeadB, kKTileBytes = X::kKTileB, kVTileBytes = X::kKTileB, kVBase = X::kVBaseB;
  // tile bases are multiples of 8 KiB from a 256-byte aligned start: the XOR constants of the swizzle (< 256)
  // never reach a tile base
  __shared__ __attribute__((aligned(256))) char smem[kBuffers * (kKTileBytes + kVTileBytes)];
  constexpr int kTileRows = WAVES * 32;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int g = lane >> 4;        // lane group: which 4 + 4 keys of a block
  const int j = lane & 15;        // row inside a row tile

  const AttnItem item = a.items[blockIdx.x];
  const AttnReq rq = a.reqs[item.req];
  const int G = a.G;
  const int P = rq.prefix;
  const int L = rq.prefix + rq.chunk;
  const int n_rows = rq.chunk * G;
  const int last_page = rq.pages - 1;

  // a wave of the second half (these copy no tiles) whose 32 rows all lie past the end of the chunk ends here
  if (wave >= WAVES / 2 && item.row0 + wave * 32 >= n_rows) return;

  // ---- this lane's two query rows: their Q fragments stay in registers for the whole KV loop
  frag qf[kSteps][2];
  bool live[2];
  int tok[2];
  int64_t orow_idx[2];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    int row = item.row0 + wave * 32 + rt * 16 + j;
    live[rt] = row < n_rows;
    row = live[rt] ? row : n_rows - 1;            // dead rows recompute the last row, never stored
    tok[rt] = row / G;
    const int qhead = item.kv_head * G + (row - tok[rt] * G);
    orow_idx[rt] = (int64_t)(rq.q_off + tok[rt]) * a.Hq + qhead;
    const char* qrow = reinterpret_cast<const char*>(a.q) + orow_idx[rt] * kRowBytes;
#pragma unroll
    for (int c = 0; c < kSteps; ++c) qf[c][rt] = *reinterpret_cast<const frag*>(qrow + c * 64 + g * 16);
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
  if (SPLIT && t_lo >= n_tiles) {
    // no key of the slice is visible to any row of the tile
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
      if (live[rt]) {
        char* orow = reinterpret_cast<char*>(a.o_parts) + ((int64_t)item.slice * a.rows_total + orow_idx[rt]) * (kD * 4);
#pragma unroll
        for (int dt = 0; dt < kDTiles; ++dt)
          *reinterpret_cast<f32x4*>(orow + (dt * 16 + g * 4) * 4) = f32x4{0.f, 0.f, 0.f, 0.f};
        if (g == 0) a.lse_parts[(int64_t)item.slice * a.rows_total + orow_idx[rt]] = -INFINITY;
      }
    return;
  }

  // ---- global -> LDS, no registers in between (as in attn_prefill.hip): one wave instruction writes
  //      1 KiB of LDS, 4 (D 64: 8) tile rows of 16 (8) granules inside one page; lane i fetches, for granule
  //      position i % kGran of row i / kGran, the logical granule (i % kGran) ^ swz(row).  The first wave of
  //      each SIMD copies.
  constexpr int kFetchWaves = WAVES / 2;
  constexpr int kChunks = kKTileBytes / 1024;                 // 1 KiB chunks per K (or V) tile
  constexpr int kFetch = kChunks / kFetchWaves;               // chunks per fetching wave
  static_assert(kChunks % kFetchWaves == 0 && kFetch <= 8, "tile must split evenly over the fetching waves");
  const char* kbase = reinterpret_cast<const char*>(a.k_pool) + (int64_t)item.kv_head * kPageHeadBytes;
  const char* vbase = reinterpret_cast<const char*>(a.v_pool) + (int64_t)item.kv_head * kPageHeadBytes;
  const int64_t page_stride = (int64_t)a.Hkv * kPageHeadBytes;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const uint32_t smem_base = (uint32_t)(uintptr_t)(MC_LDS char*)smem;
  const bool fetcher = wave_u < kFetchWaves;
  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  const_i32_ptr btc = (const_i32_ptr)(a.block_tables + (int64_t)item.req * a.max_pages);
  const int64_t first_page_off = (int64_t)btc[0] * page_stride;   // page of key 0: always valid
  int pid[kFetch];
  int pid_next[kFetch];
  auto load_ids = [&](int tile) __attribute__((always_inline)) {
    if (!fetcher) return;
#pragma unroll
    for (int i = 0; i < kFetch; ++i) {
      int lp = tile * (kTileKeys / kPageTokens) + (wave_u + i * kFetchWaves) / X::kPageChunks;
      lp = lp < last_page ? lp : last_page;                  // never index the table past the request's pages
      pid_next[i] = btc[lp];
    }
  };
  auto take_ids = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < kFetch; ++i) pid[i] = pid_next[i];
  };
  // row of the page this lane copies a granule of (the swizzles depend on the row modulo 16 only)
  const int lane_row = (wave_u % X::kPageChunks) * X::kChunkRows + lane / X::kGran;
  const uint32_t k_src = (uint32_t)(lane_row * kRowBytes + (((lane % X::kGran) ^ X::k_swz(lane_row)) << 4));
  const uint32_t v_src = (uint32_t)(lane_row * kRowBytes + (((lane % X::kGran) ^ X::v_swz(lane_row)) << 4));
  static_assert(kFetchWaves % X::kPageChunks == 0, "a fetching wave's chunks must all sit at the same rows of their pages");
  auto fetch = [&](int tile, int buf) __attribute__((always_inline)) {
    if (!fetcher) return;
    const uint32_t dst0 = smem_base + buf * kKTileBytes + wave_u * 1024;
    if ((tile + 1) * kTileKeys <= L) {
#pragma unroll
      for (int i = 0; i < kFetch; ++i) {
        const int64_t page_off = (int64_t)pid[i] * page_stride;
        const uint32_t dst = dst0 + i * kFetchWaves * 1024;
        dma16(kbase + page_off, k_src, dst);
        dma16(vbase + page_off, v_src, dst + kVBase);
      }
    } else {
      // slots at or past the request's length may hold anything: those lanes copy row 0 of the request's
      // first page instead; the causal mask hides the key
#pragma unroll
      for (int i = 0; i < kFetch; ++i) {
        const int row = (wave_u + i * kFetchWaves) * X::kChunkRows + lane / X::kGran;
        const bool in_seq = tile * kTileKeys + row < L;
        const int64_t page_off = (int64_t)pid[i] * page_stride;
        const char* ks = kbase + (in_seq ? page_off + k_src : first_page_off + (k_src & (kRowBytes - 1)));
        const char* vs = vbase + (in_seq ? page_off + v_src : first_page_off + (v_src & (kRowBytes - 1)));
        const uint32_t dst = dst0 + i * kFetchWaves * 1024;
        dma16(ks, dst);
        dma16(vs, dst + kVBase);
      }
    }
  };
  auto copies_landed = [&]() __attribute__((always_inline)) { __builtin_amdgcn_s_waitcnt(0x0F70); };

  // ---- running softmax state and output accumulators: o[dt][rt] register r = column 16 dt + 4 g + r of row 16 rt + j
  acc4 o[kDTiles][2];
  float m_run[2] = {-INFINITY, -INFINITY};   // reference of the probabilities accumulated so far (log2 units)
  // Row sums come from the matrix cores: l_acc[rt] += ones (16 x 32) . P^T (32 keys x 16 rows) leaves, in all four
  // registers of lane (j, g), the sum of row j's rounded probabilities over the whole block, lane groups included
  // (2 MFMAs per block instead of 8 dot-product instructions, which cost a matrix-pipe slot each).
  acc4 l_acc[2] = {acc4{0.f, 0.f, 0.f, 0.f}, acc4{0.f, 0.f, 0.f, 0.f}};
  frag ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;
  asm volatile("" : "+v"(ones));             // kept in registers, not rebuilt at every use
#pragma unroll
  for (int dt = 0; dt < kDTiles; ++dt)
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) o[dt][rt] = acc4{0.f, 0.f, 0.f, 0.f};
  const float c = a.scale_log2e;
  const uint32_t k_lane = smem_base + X::k_lane_off(lane);
  const uint32_t v_lane = smem_base + kVBase + X::v_lane_off(lane);
  uint32_t kx[kSteps], vx[kDTiles];
#pragma unroll
  for (int i = 0; i < kSteps; ++i) kx[i] = k_lane ^ (uint32_t)(i << 6);
#pragma unroll
  for (int i = 0; i < kDTiles; ++i) vx[i] = v_lane ^ (uint32_t)(i << 5);

  // ---- building blocks that are NOT on the steady-state path (prologue, last blocks, rare recompute)
  auto qk_block = [&](int buf, int kb, Scores& s) __attribute__((always_inline)) {
    const int off = buf * kKTileBytes + kb * 32 * kRowBytes;
    s.zero();
#pragma unroll
    for (int i = 0; i < kRing; ++i) {
      const frag kf = X::load_k(kx, off, i);
      s.t[0][i & 1] = mma(kf, qf[i >> 1][0], s.t[0][i & 1]);
      s.t[1][i & 1] = mma(kf, qf[i >> 1][1], s.t[1][i & 1]);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // Mask a block if it reaches the diagonal, take the TRUE row maxima and raise the references if some row
  // outgrew its own by more than the slack (rare, wave-uniform branch; always taken for the first block).
  auto settle_reference = [&](Scores& s, int key0, auto masked_tag) __attribute__((always_inline)) {
    constexpr bool kMasked = decltype(masked_tag)::value;
    float mx[2];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      if (kMasked) {
        // key of (kt, r): key0 + 16 kt + 4 g + r; visible iff <= P + tok
        const int lim = P + tok[rt] - key0 - 4 * g;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 4; ++r) s.t[rt][kt][r] = (16 * kt + r <= lim) ? s.t[rt][kt][r] : -INFINITY;
      }
      float m = s.t[rt][0][0];
#pragma unroll
      for (int e = 1; e < 8; ++e) m = fmaxf(m, s.t[rt][e >> 2][e & 3]);
      mx[rt] = max_over_groups(m) * c;
    }
    if (__builtin_amdgcn_ballot_w64(mx[0] > m_run[0] + kRaiseAbove || mx[1] > m_run[1] + kRaiseAbove) != 0) {
#pragma unroll
      for (int rt = 0; rt < 2; ++rt) {
        const float m_new = fmaxf(m_run[rt], mx[rt] + kRefLift);
        // a row that has seen no key yet keeps -inf (only in a slice that starts beyond the row's diagonal)
        const float alpha = (SPLIT && m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m_run[rt] - m_new);
        l_acc[rt] *= alpha;
        m_run[rt] = m_new;
#pragma unroll
        for (int dt = 0; dt < kDTiles; ++dt) o[dt][rt] *= alpha;
      }
    }
  };
  // scores -> probabilities against the references as they stand, rounded the way P V multiplies them
  auto probabilities = [&](Scores& s, PBlock& pb) __attribute__((always_inline)) {
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      const float m_ref = SPLIT ? fmaxf(m_run[rt], kNoKeyYet) : m_run[rt];
#pragma unroll
      for (int e = 8 * rt; e < 8 * rt + 8; ++e) s.set(e, __builtin_amdgcn_exp2f(__builtin_fmaf(s.get(e), c, -m_ref)));
#pragma unroll
      for (int e = 8 * rt; e < 8 * rt + 8; e += 2) round_pair(pb, s, e);
    }
  };
  auto add_row_sums = [&](const PBlock& pb) __attribute__((always_inline)) {
    l_acc[0] = mma(ones, pb.f(0), l_acc[0]);
    l_acc[1] = mma(ones, pb.f(1), l_acc[1]);
  };
  auto pv_block = [&](int buf, int kb, const PBlock& pb) __attribute__((always_inline)) {
    const int off = buf * kVTileBytes + kb * 32 * kRowBytes;
#pragma unroll
    for (int dt = 0; dt < kDTiles; ++dt) {
      const frag vf = X::load_v(vx, off, dt);
      o[dt][0] = mma(vf, pb.f(0), o[dt][0]);
      o[dt][1] = mma(vf, pb.f(1), o[dt][1]);
    }
  };

  // ---- KV loop.  Software pipeline over 32-key blocks, scheduled by hand (the order written is the order
  //      issued), around one ring of 8 fragment registers:
  //        phase A  scores of block j+1: step i multiplies ring[i] (K fragment i, read during the previous
  //                 phase B) into both row tiles and frees it; the V fragment that P V step i of block j
  //                 needs is read into the freed slot; under these MFMAs the vector ALU turns the scores of
  //                 block j into probabilities, two per step.
  //        phase B  P V of block j: step i multiplies ring[i] (the V fragment) into both row tiles and frees
  //                 it; K fragment i of block j+2 is read into the freed slot.
  frag ring[kRing];
  Scores s_cur, s_next;
  auto load_k_ring = [&](int buf, int kb) __attribute__((always_inline)) {
    const int off = buf * kKTileBytes + kb * 32 * kRowBytes;
#pragma unroll
    for (int i = 0; i < kRing; ++i) ring[i] = X::load_k(kx, off, i);
  };
  // a probability of 2 or more (or not finite) means its score outgrew the reference: the block is then
  // recomputed against its true maxima (nothing was accumulated yet)
  PBlock pb;
  auto phase_a = [&](int buf_cur, int kb_cur) __attribute__((always_inline)) {
    const int off_v = buf_cur * kVTileBytes + kb_cur * 32 * kRowBytes;
    s_cur = s_next;
    s_next.zero();
    float m_ref[2];
    constexpr int kPer = 16 / kRing;     // scores a step turns into probabilities
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) m_ref[rt] = SPLIT ? fmaxf(m_run[rt], kNoKeyYet) : m_run[rt];
#pragma unroll
    for (int i = 0; i < kRing; ++i) {
      // the step's vector work first (two exponentials; rounding and summing trail one step behind the
      // exponentials they depend on), then its two MFMAs and the fragment read: measured best of the orders tried
      const int e0 = kPer * i;
#pragma unroll
      for (int e = e0; e < e0 + kPer; ++e) s_cur.set(e, __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur.get(e), c, -m_ref[e >> 3])));
      if (i > 0) {
#pragma unroll
        for (int e = e0 - kPer; e < e0; e += 2) round_pair(pb, s_cur, e);
      }
      __builtin_amdgcn_sched_barrier(0);
      // consecutive MFMAs always share an operand register (the K fragment inside a step, the Q fragment across
      // the steps of a head_dim chunk): odd steps take the row tiles in reverse order (+1 % under the power limit)
      {
        const int ra = i & 1, rb = ra ^ 1;
        s_next.t[ra][i & 1] = mma(ring[i], qf[i >> 1][ra], s_next.t[ra][i & 1]);
        __builtin_amdgcn_sched_barrier(0);
        s_next.t[rb][i & 1] = mma(ring[i], qf[i >> 1][rb], s_next.t[rb][i & 1]);
      }
      ring[i] = X::load_v(vx, off_v, i);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int e = 16 - kPer; e < 16; e += 2) round_pair(pb, s_cur, e);
    // OR of the block's packed probabilities
    const uint32_t seen = pb.w[0][0] | pb.w[0][1] | pb.w[0][2] | pb.w[0][3] | pb.w[1][0] | pb.w[1][1] | pb.w[1][2] | pb.w[1][3];
    if (__builtin_expect(__builtin_amdgcn_ballot_w64((seen & kGuardBits) != 0) != 0, 0)) {   // (laid out behind the loop)
      qk_block(buf_cur, kb_cur, s_cur);
      settle_reference(s_cur, 0, std::false_type{});
      probabilities(s_cur, pb);
    }
  };
  auto phase_b = [&](int buf_pre, int kb_pre) __attribute__((always_inline)) {
    const int off_k = buf_pre * kKTileBytes + kb_pre * 32 * kRowBytes;
#pragma unroll
    for (int i = 0; i < kRing; ++i) {
      {
        const int ra = i & 1, rb = ra ^ 1;      // as in phase A: the V fragment inside a step, P across steps
        o[i][ra] = mma(ring[i], pb.f(ra), o[i][ra]);
        __builtin_amdgcn_sched_barrier(0);
        if (i == 0 || i == 1) {              // the row sums of the tile just used: the P operand stays where it is
          l_acc[ra] = mma(ones, pb.f(ra), l_acc[ra]);
          __builtin_amdgcn_sched_barrier(0);
        }
        o[i][rb] = mma(ring[i], pb.f(rb), o[i][rb]);
      }
      ring[i] = X::load_k(kx, off_k, i);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // one block start to finish, for the few blocks that may reach the diagonal
  auto plain_block = [&](int buf, int kb, int key0, Scores& s, bool have_scores) __attribute__((always_inline)) {
    if (!have_scores) qk_block(buf, kb, s);
    settle_reference(s, key0, std::true_type{});
    PBlock pbl;
    probabilities(s, pbl);
    add_row_sums(pbl);
    pv_block(buf, kb, pbl);
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
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  int buf = 0;
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
  const int n_plain = n_free < n_tiles - 1 ? n_free : n_tiles - 1;
  qk_block(0, 0, s_next);
  if (tile < n_plain) {
    settle_reference(s_next, 0, std::false_type{});
    load_k_ring(0, 1);
    // the two waves of a SIMD run half a step apart (see attn_prefill.hip)
    const bool late_barrier = wave_u >= WAVES / 2;
    auto pipelined_tile = [&](auto buf_tag) __attribute__((always_inline)) {
      constexpr int b = decltype(buf_tag)::value, bn = (b + 1) % kBuffers;
      buf = b;
      if (!late_barrier) tile_sync(tile);
      phase_a(b, 0);
      if (late_barrier) tile_sync(tile);
      phase_b(bn, 0);
      phase_a(b, 1);
      phase_b(bn, 1);
      buf = bn;
      ++tile;
    };
    for (;;) {
      if (tile >= n_plain) break;
      // Where the loop body sits relative to the 64-byte instruction fetch lines changes its speed by up to
      // 3.5 % (all 16 offsets measured on the 128k-context workload, with the rare recompute path laid out
      // behind the loop); pin the best one, so that edits elsewhere in the kernel cannot move it.
      asm volatile(".p2align 6");
      pipelined_tile(std::integral_constant<int, 0>{});
      if (tile >= n_plain) break;
      pipelined_tile(std::integral_constant<int, 1>{});
      if (tile >= n_plain) break;
      pipelined_tile(std::integral_constant<int, 2>{});
    }
  }
  bool have_scores = true;
  for (; tile < n_tiles; ++tile) {
    const int buf_next = buf == 2 ? 0 : buf + 1;
    tile_sync(tile);
    plain_block(buf, 0, tile * kTileKeys, s_next, have_scores);
    have_scores = false;
    plain_block(buf, 1, tile * kTileKeys + 32, s_next, false);
    buf = buf_next;
  }

  // ---- epilogue: normalise, round, store; a lane holds 4 consecutive columns per (dt, rt)
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    const float l_run = l_acc[rt][0];
    if (!live[rt]) continue;
    if (!SPLIT) {
      const float inv = 1.0f / l_run;
      char* orow = reinterpret_cast<char*>(a.out) + orow_idx[rt] * kRowBytes;
#pragma unroll
      for (int dt = 0; dt < kDTiles; ++dt) {
        bf16x4 v;
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = (__bf16)(o[dt][rt][r] * inv);
        *reinterpret_cast<bf16x4*>(orow + (dt * 16 + g * 4) * 2) = v;
      }
      if (a.lse != nullptr && g == 0)
        a.lse[orow_idx[rt]] = (m_run[rt] + __builtin_amdgcn_logf(l_run)) * 0.6931471805599453f;
    } else {
      // partial result in fp32; a row that saw no key of the slice has l = 0: zeros and -inf
      const float inv = l_run > 0.f ? 1.0f / l_run : 0.f;
      char* orow = reinterpret_cast<char*>(a.o_parts) + ((int64_t)item.slice * a.rows_total + orow_idx[rt]) * (kD * 4);
#pragma unroll
      for (int dt = 0; dt < kDTiles; ++dt)
        *reinterpret_cast<f32x4*>(orow + (dt * 16 + g * 4) * 4) =
            f32x4{o[dt][rt][0] * inv, o[dt][rt][1] * inv, o[dt][rt][2] * inv, o[dt][rt][3] * inv};
      if (g == 0)
        a.lse_parts[(int64_t)item.slice * a.rows_total + orow_idx[rt]] =
            l_run > 0.f ? (m_run[rt] + __builtin_amdgcn_logf(l_run)) * 0.6931471805599453f : -INFINITY;
    }
  }
}

}  // namespace

hipError_t launch_attn_bf16(const AttnArgs& args, hipStream_t stream) {
  (void)hipGetLastError();   // drop any stale error of earlier, unrelated runtime calls
  const bool split = args.kv_splits > 0;
  if (args.head_dim == 128) {
    if (split) attn_prefill_bf16_kernel<128, kWaves, true><<<args.n_items, kWaves * 64, 0, stream>>>(args);
    else attn_prefill_bf16_kernel<128, kWaves, false><<<args.n_items, kWaves * 64, 0, stream>>>(args);
  } else if (args.head_dim == 64) {
    if (split) attn_prefill_bf16_kernel<64, kWaves, true><<<args.n_items, kWaves * 64, 0, stream>>>(args);
    else attn_prefill_bf16_kernel<64, kWaves, false><<<args.n_items, kWaves * 64, 0, stream>>>(args);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace mc
