/*
 * CPU oracle for the KVCache-reuse hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain C, fp64, one loop per step of the definition, no tiling, no running
 * softmax, no code shared with the HIP library.  Only tests, the smoke check
 * and the benchmark's cpu_baseline leg may call this; the product path never
 * does.
 *
 * What it computes (paper Section 3, steps 1-2: a prefill node receives the
 * ids of reusable prefix blocks plus the ids of all blocks of the request and
 * finishes prefill for the rest on top of the cached prefix; Section 5.2:
 * per-layer load and store of KVCache around attention):
 *
 *   request r has P_r reused prefix tokens and C_r new tokens; chunk row i is
 *   absolute position P_r + i and sees keys j = 0 .. P_r + i (itself included);
 *   query head h reads KV head h / (Hq / Hkv);
 *   key j lives in physical page block_table[r][j / S], slot j % S.
 *
 *     s_j = scale * sum_d Q[i,h,d] * K(j)[d]
 *     m   = max_j s_j,  e_j = exp(s_j - m),  Z = sum_j e_j,  p_j = e_j / Z
 *     O[i,h,:] = sum_j p_j * V(j)[:]        LSE[i,h] = m + ln Z
 *
 * Reuse of the prefix changes nothing about the result, so this is the plain
 * definition of causal softmax attention written out; the paper prints no
 * formula and no numeric example for it.
 *
 * Pins (tests/test_oracle_*.py): reuse == full recomputation over the
 * concatenated sequence by an un-paged dense formulation; softmax rows sum to
 * one; closed forms (uniform scores -> running mean of V, constant V, first
 * row of a P = 0 request); needle keys through the block table; page
 * permutation, chunk split, GQA expansion, log-sum-exp merge of key subsets;
 * NaN in every slot the mask hides; pack followed by unpack is the identity.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { MCO_BF16 = 0, MCO_F32 = 1 };

int mco_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* exact widening of one stored element to double */
static inline double widen(const void* base, int dtype, int64_t idx) {
  if (dtype == MCO_BF16) {
    uint32_t bits = (uint32_t)((const uint16_t*)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
  }
  return (double)((const float*)base)[idx];
}

/* element index of K(j)[0] / V(j)[0] for KV head g of request r in a [N, Hkv, S, D] pool */
static inline int64_t kv_row(const int32_t* block_table_r, int64_t j, int g, int Hkv, int S, int D) {
  int64_t page = block_table_r[j / S];
  return ((page * Hkv + g) * S + (j % S)) * (int64_t)D;
}

/*
 * One output row.  Keys are restricted to [key_lo, key_hi) intersected with
 * the visible range [0, P + i]; the full row uses key_lo = 0, key_hi = INT64_MAX.
 * `s` is scratch for at least P + i + 1 doubles.  An empty key set gives
 * O = 0, LSE = -inf, psum = 0.
 */
static void attn_row(int dtype, const void* q, const void* k_pool, const void* v_pool,
                     const int32_t* bt_r, int64_t q_row, int P, int i, int h, int Hq, int Hkv, int D,
                     int S, double scale, int64_t key_lo, int64_t key_hi, double* s, double* o,
                     double* lse, double* psum) {
  const int G = Hq / Hkv;
  const int g = h / G;
  int64_t lo = key_lo < 0 ? 0 : key_lo;
  int64_t hi = (int64_t)P + i + 1;
  if (key_hi < hi) hi = key_hi;
  for (int d = 0; d < D; ++d) o[d] = 0.0;
  if (hi <= lo) {
    *lse = -INFINITY;
    if (psum) *psum = 0.0;
    return;
  }
  const int64_t qbase = (q_row * Hq + h) * (int64_t)D;
  /* scores */
  double m = -INFINITY;
  for (int64_t j = lo; j < hi; ++j) {
    const int64_t kb = kv_row(bt_r, j, g, Hkv, S, D);
    double acc = 0.0;
    for (int d = 0; d < D; ++d) acc += widen(q, dtype, qbase + d) * widen(k_pool, dtype, kb + d);
    acc *= scale;
    s[j - lo] = acc;
    if (acc > m) m = acc;
  }
  /* softmax */
  double Z = 0.0;
  for (int64_t j = lo; j < hi; ++j) {
    s[j - lo] = exp(s[j - lo] - m);
    Z += s[j - lo];
  }
  double ps = 0.0;
  for (int64_t j = lo; j < hi; ++j) {
    s[j - lo] /= Z;
    ps += s[j - lo];
  }
  /* weighted sum of V rows */
  for (int64_t j = lo; j < hi; ++j) {
    const int64_t vb = kv_row(bt_r, j, g, Hkv, S, D);
    const double p = s[j - lo];
    for (int d = 0; d < D; ++d) o[d] += p * widen(v_pool, dtype, vb + d);
  }
  *lse = m + log(Z);
  if (psum) *psum = ps;
}

/*
 * Selected rows.  rows[3*n] holds (request, query head, chunk row) triples.
 * key_lo / key_hi may be NULL (full visible range) or hold one bound per row.
 * out [n, D] fp64, lse [n] fp64, psum [n] fp64 or NULL (sum of the row's
 * probabilities).  Returns 0, or -1 on a bad argument (nothing written).
 */
int mco_attn_rows(int dtype, const void* q, const void* k_pool, const void* v_pool,
                  const int32_t* block_tables, int max_pages_per_req, const int32_t* prefix_lens,
                  const int32_t* new_lens, int batch, int Hq, int Hkv, int D, int S, double scale,
                  int64_t n, const int32_t* rows, const int64_t* key_lo, const int64_t* key_hi,
                  double* out, double* lse, double* psum) {
  if (Hkv <= 0 || Hq % Hkv != 0 || D <= 0 || S <= 0) return -1;
  int64_t* q_off = (int64_t*)malloc(sizeof(int64_t) * (size_t)(batch + 1));
  if (!q_off) return -1;
  q_off[0] = 0;
  for (int r = 0; r < batch; ++r) q_off[r + 1] = q_off[r] + new_lens[r];
  for (int64_t t = 0; t < n; ++t) {
    int r = rows[3 * t], h = rows[3 * t + 1], i = rows[3 * t + 2];
    if (r < 0 || r >= batch || h < 0 || h >= Hq || i < 0 || i >= new_lens[r] ||
        (int64_t)max_pages_per_req * S < (int64_t)prefix_lens[r] + new_lens[r]) {
      free(q_off);
      return -1;
    }
  }
  int failed = 0;
#pragma omp parallel
  {
    double* s = NULL;
    int64_t cap = 0;
#pragma omp for schedule(dynamic, 1)
    for (int64_t t = 0; t < n; ++t) {
      int r = rows[3 * t], h = rows[3 * t + 1], i = rows[3 * t + 2];
      int64_t need = (int64_t)prefix_lens[r] + i + 1;
      if (need > cap) {
        free(s);
        s = (double*)malloc(sizeof(double) * (size_t)need);
        cap = s ? need : 0;
      }
      if (!s) {
        failed = 1;
        continue;
      }
      attn_row(dtype, q, k_pool, v_pool, block_tables + (int64_t)r * max_pages_per_req, q_off[r] + i,
               prefix_lens[r], i, h, Hq, Hkv, D, S, scale, key_lo ? key_lo[t] : 0,
               key_hi ? key_hi[t] : INT64_MAX, s, out + t * D, lse + t, psum ? psum + t : NULL);
    }
    free(s);
  }
  free(q_off);
  return failed ? -1 : 0;
}

/*
 * Every row of every request: out [total_new, Hq, D] fp64, lse [total_new, Hq]
 * fp64, psum same shape as lse or NULL.
 */
int mco_prefill_attn_paged(int dtype, const void* q, const void* k_pool, const void* v_pool,
                           const int32_t* block_tables, int max_pages_per_req,
                           const int32_t* prefix_lens, const int32_t* new_lens, int batch, int Hq,
                           int Hkv, int D, int S, double scale, double* out, double* lse,
                           double* psum) {
  int64_t total = 0;
  for (int r = 0; r < batch; ++r) total += new_lens[r];
  int64_t n = total * Hq;
  if (n == 0) return 0;
  int32_t* rows = (int32_t*)malloc(sizeof(int32_t) * 3 * (size_t)n);
  if (!rows) return -1;
  int64_t t = 0;
  for (int r = 0; r < batch; ++r)
    for (int i = 0; i < new_lens[r]; ++i)
      for (int h = 0; h < Hq; ++h) {
        rows[3 * t] = r;
        rows[3 * t + 1] = h;
        rows[3 * t + 2] = i;
        ++t;
      }
  int rc = mco_attn_rows(dtype, q, k_pool, v_pool, block_tables, max_pages_per_req, prefix_lens,
                         new_lens, batch, Hq, Hkv, D, S, scale, n, rows, NULL, NULL, out, lse, psum);
  free(rows);
  return rc;
}

/*
 * Layer-wise store path (Section 5.2): gather the listed pages of one layer's
 * scattered pool into a contiguous buffer, in list order, each page verbatim.
 */
int mco_kv_pack_layer(const uint8_t* k_pool, const uint8_t* v_pool, int64_t num_pages,
                      int64_t page_bytes, const int32_t* page_ids, int64_t n, uint8_t* k_out,
                      uint8_t* v_out, int threads) {
  for (int64_t i = 0; i < n; ++i)
    if (page_ids[i] < 0 || page_ids[i] >= num_pages) return -1;
#pragma omp parallel for num_threads(threads > 0 ? threads : 1) schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    memcpy(k_out + i * page_bytes, k_pool + (int64_t)page_ids[i] * page_bytes, (size_t)page_bytes);
    memcpy(v_out + i * page_bytes, v_pool + (int64_t)page_ids[i] * page_bytes, (size_t)page_bytes);
  }
  return 0;
}

/*
 * Layer-wise load path: scatter a contiguous buffer of n pages into the
 * listed (unique) pages of a pool; pages not listed keep their bytes.
 */
int mco_kv_unpack_layer(const uint8_t* k_in, const uint8_t* v_in, int64_t num_pages,
                        int64_t page_bytes, const int32_t* page_ids, int64_t n, uint8_t* k_pool,
                        uint8_t* v_pool, int threads) {
  for (int64_t i = 0; i < n; ++i)
    if (page_ids[i] < 0 || page_ids[i] >= num_pages) return -1;
#pragma omp parallel for num_threads(threads > 0 ? threads : 1) schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    memcpy(k_pool + (int64_t)page_ids[i] * page_bytes, k_in + i * page_bytes, (size_t)page_bytes);
    memcpy(v_pool + (int64_t)page_ids[i] * page_bytes, v_in + i * page_bytes, (size_t)page_bytes);
  }
  return 0;
}

/*
 * Incremental prefill keeps the KVCache of the tokens it has just computed (Section 3, step 2):
 * token i of request r (absolute position P_r + i) goes to slot (P_r + i) % S of page
 * block_table[r][(P_r + i) / S], for every KV head, bytes verbatim.  k_new / v_new are
 * [total_new, Hkv, row_bytes], pools are [N, Hkv, S, row_bytes].  Slots not written keep
 * their bytes.  Returns -1 on a bad argument (nothing written).
 */
int mco_kv_append_paged(const uint8_t* k_new, const uint8_t* v_new, uint8_t* k_pool, uint8_t* v_pool,
                        int64_t num_pages, const int32_t* block_tables, int max_pages_per_req,
                        const int32_t* prefix_lens, const int32_t* new_lens, int batch, int Hkv, int S,
                        int64_t row_bytes) {
  for (int r = 0; r < batch; ++r) {
    if (prefix_lens[r] < 0 || new_lens[r] < 0) return -1;
    if (new_lens[r] > 0 && (int64_t)max_pages_per_req * S < (int64_t)prefix_lens[r] + new_lens[r]) return -1;
    for (int i = 0; i < new_lens[r]; ++i) {
      int64_t page = block_tables[(int64_t)r * max_pages_per_req + (prefix_lens[r] + i) / S];
      if (page < 0 || page >= num_pages) return -1;
    }
  }
  int64_t t = 0;
  for (int r = 0; r < batch; ++r)
    for (int i = 0; i < new_lens[r]; ++i, ++t) {
      const int64_t pos = (int64_t)prefix_lens[r] + i;
      const int64_t page = block_tables[(int64_t)r * max_pages_per_req + pos / S];
      for (int g = 0; g < Hkv; ++g) {
        const int64_t dst = ((page * Hkv + g) * S + pos % S) * row_bytes;
        const int64_t src = (t * Hkv + g) * row_bytes;
        memcpy(k_pool + dst, k_new + src, (size_t)row_bytes);
        memcpy(v_pool + dst, v_new + src, (size_t)row_bytes);
      }
    }
  return 0;
}

/*
 * Merge of partial attention results over disjoint key subsets (Section 5.1: sequence
 * parallelism rests on the attention operator being associative over slices of the keys).
 * Part s holds, for every row, the softmax-weighted V sum over ITS keys, o_parts[s][row][:],
 * and the log of its exponential sum, lse_parts[s][row] (natural log; -inf = the part saw no
 * key of that row).  The whole row is
 *     lse = log sum_s exp(lse_s),   out = sum_s exp(lse_s - lse) * o_s,
 * written out as that definition with the usual shift by the largest lse_s.  A row none of
 * whose parts saw a key gives out = 0, lse = -inf.  Partials are fp32, results fp64.
 */
int mco_attn_merge_lse(const float* o_parts, const float* lse_parts, int n_parts, int64_t rows, int D,
                       double* out, double* lse) {
  if (n_parts < 0 || rows < 0 || D < 0) return -1;
  for (int64_t t = 0; t < rows; ++t) {
    double m = -INFINITY;
    for (int s = 0; s < n_parts; ++s) {
      const double l = (double)lse_parts[(int64_t)s * rows + t];
      if (l > m) m = l;
    }
    for (int d = 0; d < D; ++d) out[t * D + d] = 0.0;
    if (m == -INFINITY) {
      lse[t] = -INFINITY;
      continue;
    }
    double Z = 0.0;
    for (int s = 0; s < n_parts; ++s) Z += exp((double)lse_parts[(int64_t)s * rows + t] - m);
    for (int s = 0; s < n_parts; ++s) {
      const double w = exp((double)lse_parts[(int64_t)s * rows + t] - m) / Z;
      if (w == 0.0) continue;   /* a part without keys may hold anything, NaN included */
      for (int d = 0; d < D; ++d) out[t * D + d] += w * (double)o_parts[((int64_t)s * rows + t) * D + d];
    }
    lse[t] = m + log(Z);
  }
  return 0;
}

/*
 * Prefix block keys (Section 6.1 / Algorithm 1, PrefixHash; Figure "KVCache pool": a block's
 * hash value is determined by its own hash and by its prefix).  The paper fixes the block size
 * (512 tokens) but not the hash; the reading taken here, in 64-bit wrap-around arithmetic:
 *
 *   mix(x)      = the splitmix64 output function: x += 0x9E3779B97F4A7C15;
 *                 x = (x ^ x >> 30) * 0xBF58476D1CE4E5B9; x = (x ^ x >> 27) * 0x94D049BB133111EB;
 *                 x ^ x >> 31
 *   digest(b)   = mix( n_b + sum_j mix( (uint64) token_j  +  (j << 32) ) ),  j = 0 .. n_b - 1 inside
 *                 block b, n_b = its token count (a block's OWN hash: position-salted, hence
 *                 order-sensitive; a plain sum, so it can be formed in any order)
 *   key(0)      = mix( digest(0) ^ 0x243F6A8885A308D3 )
 *   key(b)      = mix( digest(b) ^ rotl(key(b-1), 23) * 0x9E3779B97F4A7C15 )     (the prefix enters)
 *
 * Every block gets a key, the last one of a request may be partial (the two request samples
 * the paper prints in Section 4 carry ceil(input_length / 512) ids): request r has
 * ceil(len_r / B) keys, written back to back.  tok_offsets has batch + 1 entries.  Returns the
 * number of keys, or -1 on a bad argument.
 */
static uint64_t mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

uint64_t mco_mix64(uint64_t x) { return mix64(x); }

int64_t mco_prefix_hash(const int32_t* tokens, const int64_t* tok_offsets, int batch, int block_tokens,
                        uint64_t* keys) {
  if (batch < 0 || block_tokens <= 0) return -1;
  for (int r = 0; r < batch; ++r)
    if (tok_offsets[r + 1] < tok_offsets[r]) return -1;
  int64_t n = 0;
  for (int r = 0; r < batch; ++r) {
    const int32_t* t = tokens + tok_offsets[r];
    const int64_t len = tok_offsets[r + 1] - tok_offsets[r];
    const int64_t blocks = (len + block_tokens - 1) / block_tokens;
    uint64_t prev = 0;
    for (int64_t b = 0; b < blocks; ++b) {
      const int64_t nb = len - b * block_tokens < block_tokens ? len - b * block_tokens : block_tokens;
      uint64_t sum = (uint64_t)nb;
      for (int64_t j = 0; j < nb; ++j)
        sum += mix64((uint64_t)(uint32_t)t[b * block_tokens + j] + ((uint64_t)j << 32));
      const uint64_t digest = mix64(sum);
      const uint64_t key = b == 0 ? mix64(digest ^ 0x243F6A8885A308D3ull)
                                  : mix64(digest ^ (((prev << 23) | (prev >> 41)) * 0x9E3779B97F4A7C15ull));
      keys[n++] = key;
      prev = key;
    }
  }
  return n;
}

/*
 * Longest prefix match of every request against every prefill instance's cache keys
 * (Algorithm 1, FindBestPrefixMatch: the request's block keys are compared one by one against
 * the instance's cache keys).  prefix_len[r][i] = number of LEADING keys of request r that
 * instance i holds (the first key it does not hold ends the match); best_len[r] = the largest of
 * them, best_inst[r] = the lowest instance index that attains it (-1 if n_inst == 0).
 * Plain scans: every request key against every cache key of the instance, in order.
 */
int mco_prefix_match(const uint64_t* keys, const int64_t* key_offsets, int batch, const uint64_t* cache_keys,
                     const int64_t* cache_offsets, int n_inst, int32_t* prefix_len, int32_t* best_len,
                     int32_t* best_inst) {
  if (batch < 0 || n_inst < 0) return -1;
  for (int r = 0; r < batch; ++r) {
    best_len[r] = 0;
    best_inst[r] = n_inst > 0 ? 0 : -1;
    for (int i = 0; i < n_inst; ++i) {
      int32_t len = 0;
      for (int64_t b = key_offsets[r]; b < key_offsets[r + 1]; ++b) {
        int found = 0;
        for (int64_t c = cache_offsets[i]; c < cache_offsets[i + 1] && !found; ++c) found = cache_keys[c] == keys[b];
        if (!found) break;
        ++len;
      }
      prefix_len[(int64_t)r * n_inst + i] = len;
      if (len > best_len[r]) {
        best_len[r] = len;
        best_inst[r] = i;
      }
    }
  }
  return 0;
}
