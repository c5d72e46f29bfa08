/*
 * mc.h - C ABI of the MI355X (gfx950) KVCache-reuse hot path.
 *
 * Three operations behind Mooncake's KVCache reuse, as the paper states the
 * problem (it gives no kernel design):
 *
 *   - a prefill node is handed the ids of the prefix blocks it may reuse and of
 *     all blocks of the request, loads the former and computes prefill for the
 *     uncached tokens only, reading the reused prefix, in chunks no longer than
 *     prefill_chunk (Section 3, steps 1 and 2; Section 5.1);
 *   - per layer, KVCache is loaded before that layer's attention and stored
 *     after it, asynchronously, overlapped with compute (Section 5.2;
 *     Section 3, step 3).
 *
 * Conventions for every entry point:
 *   - "dev" pointers are device memory of the current HIP device, "host"
 *     pointers are ordinary host memory.  The caller owns every buffer; the
 *     library never allocates or frees device memory.
 *   - All device work is enqueued on `hip_stream` (a hipStream_t passed as
 *     void*; NULL = the default stream) and the call returns at once.
 *     Host arrays are read before the call returns and may be freed then.
 *   - Arguments are validated on the host first.  On any status other than
 *     MC_OK and MC_ERR_HIP nothing has been launched and no output has been
 *     touched.  MC_ERR_HIP means the HIP runtime refused a step of the call:
 *     steps of the same call that were enqueued before it (an upload, a copy,
 *     the first of two kernels) stay enqueued, so the outputs are undefined.
 *   - The calls that take host lengths or offsets and hand them to a kernel
 *     (mc_prefill_attn_paged, _paged_split, _auto, _prepare, mc_kv_append_paged,
 *     mc_prefix_hash, mc_prefix_match) upload them from a small ring of pinned
 *     HOST slots the library owns.  Such a call may allocate a slot with
 *     hipHostMalloc (the first calls, or a list larger than any before), and
 *     with 256 uploads in flight it waits for the oldest: these calls are not
 *     for stream capture.  The run calls (mc_prefill_attn_run, _run_split,
 *     mc_kv_append_run), pack / unpack and the merge upload nothing, allocate
 *     nothing and never wait.  Calls may come from several host threads.
 *   - Page ids that live in device memory cannot be range-checked without a
 *     sync: an id outside [0, num_pages) is undefined behaviour.
 *   - No exceptions cross this boundary.
 */
#ifndef MC_H_
#define MC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MC_OK = 0,
  MC_ERR_NULL = 1,        /* a required pointer is NULL */
  MC_ERR_SHAPE = 2,       /* negative size, Hq % Hkv != 0, block table too short for P + C */
  MC_ERR_UNSUPPORTED = 3, /* head_dim / page_size / dtype combination with no kernel */
  MC_ERR_ALIGN = 4,       /* pointer not 16-byte aligned, or page_bytes % 16 != 0 */
  MC_ERR_RANGE = 5,       /* a size exceeds what the kernels index with 32 bits */
  MC_ERR_WORKSPACE = 6,   /* workspace NULL or smaller than mc_prefill_attn_workspace_bytes */
  MC_ERR_HIP = 7          /* the HIP runtime refused a copy or a launch */
} mc_status;

typedef enum { MC_DTYPE_BF16 = 0, MC_DTYPE_F32 = 1 } mc_dtype;

typedef struct {
  int32_t num_q_heads;  /* Hq */
  int32_t num_kv_heads; /* Hkv, divides Hq; query head h reads KV head h / (Hq / Hkv) */
  int32_t head_dim;     /* D: 128 or 64 for bf16, 64 for f32 (one row = 256 or 128 bytes) */
  int32_t page_size;    /* S tokens per page: 16 */
  int64_t num_pages;    /* N pages in each pool */
  int32_t dtype;        /* mc_dtype of Q, K, V and O */
  float softmax_scale;  /* 0 selects 1 / sqrt(head_dim) */
} mc_attn_params;

/* Human-readable name of a status code (static storage). */
const char* mc_status_string(mc_status s);

/*
 * Bytes of device workspace mc_prefill_attn_paged needs for a batch of
 * `batch` requests with `total_new_tokens` new tokens in all (the per-tile
 * work list the kernel walks).  Returns 0 for invalid arguments.
 */
size_t mc_prefill_attn_workspace_bytes(const mc_attn_params* p, int32_t batch,
                                       int64_t total_new_tokens);

/*
 * Prefix-reused, paged, chunked-prefill attention (Section 3 steps 1-2).
 *
 * Request r has P_r = prefix_lens[r] tokens whose K/V pages were reused and
 * C_r = new_lens[r] new tokens; the K/V of the new tokens are already in
 * their pages.  Row i of the request's chunk is absolute position P_r + i
 * and attends to keys 0 .. P_r + i (itself included); all prefix keys are
 * visible to every row.  Key j of request r is
 * pool[block_tables[r][j / S]][h / (Hq/Hkv)][j % S][:].
 *
 *   out[i,h,:] = sum_j softmax_j(scale * q[i,h,:] . K(j)) * V(j)
 *   lse[i,h]   = log sum_j exp(scale * q[i,h,:] . K(j))          (natural log)
 *
 *   q            dev  [total_new_tokens, Hq, D]   requests back to back
 *   k_pool       dev  [N, Hkv, S, D]              this layer's K pages
 *   v_pool       dev  [N, Hkv, S, D]
 *   block_tables dev  [batch, max_pages_per_req]  int32 logical -> physical page
 *   prefix_lens  host [batch]  P_r >= 0, need not be a multiple of S
 *   new_lens     host [batch]  C_r >= 0 (0 = the request has no rows)
 *   out          dev  [total_new_tokens, Hq, D]   dtype of q, every row written
 *   lse          dev  [total_new_tokens, Hq] fp32, or NULL
 *   workspace    dev  >= mc_prefill_attn_workspace_bytes(...), 16-byte aligned;
 *                     in use until the enqueued work has finished.  A workspace of at least
 *                     mc_prefill_attn_auto_workspace_bytes(...) lets the call run over key slices
 *                     + merge (as mc_prefill_attn_auto does) whenever whole rows would leave
 *                     compute units idle: a small chunk behind a long prefix, or a number of work
 *                     items just above a multiple of the 256 compute units.  The result is the
 *                     same to the tolerance of the two forms, not bit for bit; callers that need
 *                     one fixed form pass the minimal workspace (always whole rows) or call
 *                     mc_prefill_attn_paged_split themselves.
 *
 * Token slots at or beyond P_r + C_r in a request's last page, and pages the
 * block tables do not name, are never read as values (they may hold NaN).
 * bf16: products on the matrix cores, fp32 accumulation and softmax, output
 * rounded to nearest even.  f32: fp32 throughout.
 * batch == 0 or total_new_tokens == 0 is MC_OK and enqueues nothing.
 */
mc_status mc_prefill_attn_paged(const mc_attn_params* p, const void* q, const void* k_pool,
                                const void* v_pool, const int32_t* block_tables,
                                int32_t max_pages_per_req, const int32_t* prefix_lens,
                                const int32_t* new_lens, int32_t batch, void* out, float* lse,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Split form of mc_prefill_attn_paged for chunks too small to fill the GPU against a long
 * prefix, and the single exchange step of sequence-parallel prefill (Section 5.1: the attention
 * operator is associative over slices of the keys).
 *
 * The keys of request r are cut into kv_splits slices of whole 64-key tiles,
 * T_r = ceil(ceil((P_r + C_r) / 64) / kv_splits) tiles each: slice s covers keys
 * [64 s T_r, min(64 (s + 1) T_r, P_r + C_r)); trailing slices may be empty.  For every slice s
 * and output row (i, h) the call writes the PARTIAL result over the keys of the slice that the
 * row may see:
 *
 *   o_parts[s][i][h][:]  fp32  softmax-weighted V sum over those keys (0 if there are none)
 *   lse_parts[s][i][h]   fp32  natural log of their exponential sum    (-inf if there are none)
 *
 *   o_parts    dev  [kv_splits, total_new_tokens, Hq, D] fp32, 16-byte aligned
 *   lse_parts  dev  [kv_splits, total_new_tokens, Hq]    fp32
 *   workspace  dev  >= mc_prefill_attn_split_workspace_bytes(...)
 *
 * Everything else as mc_prefill_attn_paged.  kv_splits outside [1, MC_MAX_KV_SPLITS] is
 * MC_ERR_SHAPE.  mc_attn_merge_lse turns the partials into the whole-row result.
 */
#define MC_MAX_KV_SPLITS 256
size_t mc_prefill_attn_split_workspace_bytes(const mc_attn_params* p, int32_t batch,
                                             int64_t total_new_tokens, int32_t kv_splits);
mc_status mc_prefill_attn_paged_split(const mc_attn_params* p, const void* q, const void* k_pool,
                                      const void* v_pool, const int32_t* block_tables,
                                      int32_t max_pages_per_req, const int32_t* prefix_lens,
                                      const int32_t* new_lens, int32_t batch, int32_t kv_splits,
                                      float* o_parts, float* lse_parts, void* workspace,
                                      size_t workspace_bytes, void* hip_stream);

/*
 * Number of key slices that fills the GPU for this batch (Section 5.1: long contexts are cut so
 * that more compute can work on one request).  With n work items in the whole-row form (one per
 * request, KV head and tile of stacked query rows) and 256 compute units, s slices take
 * ceil(n s / 256) / s rounds of the whole-row item length, and every slice beyond the first adds
 * about 1 % for the partial results: the count with the least cost wins, among those that leave
 * every slice of the longest request at least 8 tiles of 64 keys and do not exceed
 * MC_MAX_KV_SPLITS.  1 means mc_prefill_attn_paged is the better call (always so from 1024 work
 * items on).  Host arithmetic only: no GPU call, nothing enqueued.  Returns 0 for arguments
 * mc_prefill_attn_paged would reject as MC_ERR_NULL / MC_ERR_SHAPE / MC_ERR_UNSUPPORTED.
 *
 *   prefix_lens, new_lens  HOST [batch]
 */
int32_t mc_prefill_attn_suggest_kv_splits(const mc_attn_params* p, const int32_t* prefix_lens,
                                          const int32_t* new_lens, int32_t batch);

/*
 * mc_prefill_attn_paged with the choice between the whole-row form and key slices + merge made
 * by the library: it takes the slice count mc_prefill_attn_suggest_kv_splits gives for the
 * lengths and, when that is above 1, runs mc_prefill_attn_paged_split and mc_attn_merge_lse on
 * partial buffers it places in the workspace.  Same arguments, same result (to the tolerance of
 * the two forms) as mc_prefill_attn_paged; the workspace is larger:
 *
 *   workspace  dev  >= mc_prefill_attn_auto_workspace_bytes(...) for the same params and lengths
 *                   (work list + request table + kv_splits * rows * (head_dim + 1) floats),
 *                   16-byte aligned; 0 is returned for arguments the call would reject
 */
size_t mc_prefill_attn_auto_workspace_bytes(const mc_attn_params* p, const int32_t* prefix_lens,
                                            const int32_t* new_lens, int32_t batch);
mc_status mc_prefill_attn_auto(const mc_attn_params* p, const void* q, const void* k_pool, const void* v_pool,
                               const int32_t* block_tables, int32_t max_pages_per_req,
                               const int32_t* prefix_lens, const int32_t* new_lens, int32_t batch, void* out,
                               float* lse, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * mc_prefill_attn_paged for callers that cannot allocate: code under HIP graph capture, serving
 * loops and harnesses that forbid hipMalloc.  Same arguments without the workspace, same result
 * (the same kernel over the same work list).  The work list and request table live in a fixed
 * device array inside the library (MC_NOALLOC_MAX_ITEMS * 16 + MC_NOALLOC_MAX_BATCH * 16 bytes
 * = 514 KiB per GPU, held until the process ends) and are built ON the device by a small kernel
 * that receives the lengths as a kernel argument: the call allocates nothing (device, pinned or
 * host heap), uploads nothing and never waits; it enqueues two kernels on `hip_stream`.
 *
 * Limits: batch <= MC_NOALLOC_MAX_BATCH and at most MC_NOALLOC_MAX_ITEMS work items
 * (sum over requests of Hkv * ceil(C_r * Hq / Hkv / 256)); beyond them the call returns
 * MC_ERR_RANGE and enqueues nothing.  Every call on a GPU uses that GPU's one array: calls whose
 * device work may overlap (different streams without an ordering between them) race on it; calls
 * on one stream, or ordered by events, are safe.  The first call on a device looks the array's
 * address up (hipGetSymbolAddress) and should be made outside stream capture.
 */
#define MC_NOALLOC_MAX_BATCH 128
#define MC_NOALLOC_MAX_ITEMS 32768
mc_status mc_prefill_attn_paged_noalloc(const mc_attn_params* p, const void* q, const void* k_pool,
                                        const void* v_pool, const int32_t* block_tables,
                                        int32_t max_pages_per_req, const int32_t* prefix_lens,
                                        const int32_t* new_lens, int32_t batch, void* out, float* lse,
                                        void* hip_stream);

/*
 * Prepare once, run per layer.  The work list and the request table depend on the lengths of the
 * batch only, and a prefill pass makes the same attention and append calls for every layer of
 * the model (Section 5.2: layer-wise prefill): mc_prefill_attn_prepare builds them and enqueues
 * their upload into the workspace ONCE; the run calls then only launch kernels - no host
 * work beyond argument checks, no upload, and nothing a stream capture could not record.
 *
 *   kv_splits  0: plan for mc_prefill_attn_run;  1 .. MC_MAX_KV_SPLITS: for mc_prefill_attn_run_split
 *   workspace  dev  >= mc_prefill_attn_workspace_bytes(...) (kv_splits == 0) or
 *                   >= mc_prefill_attn_split_workspace_bytes(...); the runs read it, so it must
 *                   keep its bytes for as long as the plan is in use, and the runs must be
 *                   ordered after the prepare call (same stream, or an event)
 *   plan       HOST out: plain data the run calls take back; valid with these params only
 *
 * The run calls compute exactly what mc_prefill_attn_paged / mc_prefill_attn_paged_split /
 * mc_kv_append_paged compute for the lengths the plan was prepared with (those calls are
 * prepare + run in one), with the same argument rules; block tables need at least
 * plan->need_pages columns.  A plan for no new tokens is empty and its runs enqueue nothing.
 * mc_kv_append_run takes either form of plan.
 */
typedef struct {
  int32_t n_items;            /* work items (workgroups) of the attention launch */
  int32_t batch;
  int32_t kv_splits;          /* 0 = whole-row form */
  int32_t need_pages;         /* most pages any request with new tokens spans */
  int64_t total_new_tokens;
  int64_t reqs_offset;        /* byte offset of the request table in the workspace */
  int32_t num_q_heads, num_kv_heads, dtype, reserved;   /* of the params it was prepared with */
} mc_attn_plan;

mc_status mc_prefill_attn_prepare(const mc_attn_params* p, const int32_t* prefix_lens, const int32_t* new_lens,
                                  int32_t batch, int32_t kv_splits, void* workspace, size_t workspace_bytes,
                                  void* hip_stream, mc_attn_plan* plan);
mc_status mc_prefill_attn_run(const mc_attn_params* p, const mc_attn_plan* plan, const void* q, const void* k_pool,
                              const void* v_pool, const int32_t* block_tables, int32_t max_pages_per_req, void* out,
                              float* lse, const void* workspace, void* hip_stream);
mc_status mc_prefill_attn_run_split(const mc_attn_params* p, const mc_attn_plan* plan, const void* q,
                                    const void* k_pool, const void* v_pool, const int32_t* block_tables,
                                    int32_t max_pages_per_req, float* o_parts, float* lse_parts,
                                    const void* workspace, void* hip_stream);
mc_status mc_kv_append_run(const mc_attn_params* p, const mc_attn_plan* plan, const void* k_new, const void* v_new,
                           void* k_pool, void* v_pool, const int32_t* block_tables, int32_t max_pages_per_req,
                           const void* workspace, void* hip_stream);

/*
 * The work list the two attention calls above launch for these lengths, in launch order, written
 * to HOST memory - for inspection and for tests of the host logic; no GPU call, nothing enqueued.
 * One work item = one workgroup = one tile of 256 stacked query rows (row = token * G + head in
 * group) of one (request, KV head), and for the split form one key slice of it:
 *
 *   items[i] = { request, kv_head, first stacked row of the tile, key slice (0 if whole-row) }
 *
 * Order: items are keyed by the keys their last row sees (split form: by the keys of the slice),
 * kept in 8 lists by (request * Hkv + kv_head + slice) mod 8, longest first within a list, and
 * dealt out round-robin - consecutive workgroups land on different XCDs, so each XCD's L2 keeps
 * the K/V stream of one (request, KV head), and the longest items start first.
 *
 *   kv_splits  0 = mc_prefill_attn_paged, 1 .. MC_MAX_KV_SPLITS = mc_prefill_attn_paged_split
 *   items      HOST int32 [capacity][4], or NULL (capacity 0) to count only
 *   n_items    HOST out: the number of work items (set whenever the status is MC_OK or
 *              MC_ERR_WORKSPACE)
 *
 * Status: what the attention call would answer to the same params and lengths (MC_ERR_NULL,
 * MC_ERR_SHAPE, MC_ERR_UNSUPPORTED, MC_ERR_RANGE); MC_ERR_WORKSPACE when capacity < n_items
 * (nothing written to items then).
 */
mc_status mc_prefill_attn_plan(const mc_attn_params* p, const int32_t* prefix_lens, const int32_t* new_lens,
                               int32_t batch, int32_t kv_splits, int32_t* items, int64_t capacity,
                               int64_t* n_items);

/*
 * Merge of partial attention results over disjoint key subsets (Section 5.1), whoever produced
 * them (mc_prefill_attn_paged_split, or other GPUs holding other slices of the sequence):
 *
 *   lse[t]    = log sum_s exp(lse_parts[s][t])
 *   out[t][:] = sum_s exp(lse_parts[s][t] - lse[t]) * o_parts[s][t][:]
 *
 *   o_parts    dev  [kv_splits, rows, head_dim] fp32
 *   lse_parts  dev  [kv_splits, rows] fp32; -inf marks a part without keys: weight 0, its
 *                   o_parts row is not read
 *   out        dev  [rows, head_dim] of `dtype` (bf16: rounded to nearest even)
 *   lse        dev  [rows] fp32, or NULL
 *
 * A row whose parts are all -inf gives out = 0, lse = -inf.  (head_dim, dtype) must be
 * (128, MC_DTYPE_BF16), (64, MC_DTYPE_BF16) or (64, MC_DTYPE_F32).  rows == 0 is MC_OK and enqueues nothing.
 */
mc_status mc_attn_merge_lse(const float* o_parts, const float* lse_parts, int32_t kv_splits, int64_t rows,
                            int32_t head_dim, int32_t dtype, void* out, float* lse, void* hip_stream);

/*
 * Bytes of device workspace mc_kv_append_paged needs (the per-request table).  0 for batch < 0.
 */
size_t mc_kv_append_workspace_bytes(int32_t batch);

/*
 * Store the new chunk's K/V into the request's pages (Section 3, step 2: incremental prefill
 * keeps the newly generated KVCache; this is what puts it where mc_prefill_attn_paged reads it).
 * Token i of request r (absolute position P_r + i) is written, for every KV head g, to
 * pool[block_tables[r][(P_r + i) / S]][g][(P_r + i) % S][:], bytes verbatim.
 *
 *   k_new, v_new  dev  [total_new_tokens, Hkv, D]  requests back to back, dtype p->dtype
 *   k_pool,v_pool dev  [N, Hkv, S, D]              written in place; other slots keep their bytes
 *   block_tables  dev  [batch, max_pages_per_req]
 *   prefix_lens, new_lens  host [batch]
 *   workspace     dev  >= mc_kv_append_workspace_bytes(batch), 16-byte aligned
 *
 * Same shape restrictions and status codes as mc_prefill_attn_paged (num_q_heads is only
 * checked for divisibility).  Two requests whose block tables name the same page for
 * positions both write: undefined which wins.
 */
mc_status mc_kv_append_paged(const mc_attn_params* p, const void* k_new, const void* v_new, void* k_pool,
                             void* v_pool, const int32_t* block_tables, int32_t max_pages_per_req,
                             const int32_t* prefix_lens, const int32_t* new_lens, int32_t batch,
                             void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Store path of layer-wise prefill (Section 5.2): gather pages of one layer's
 * scattered pools into contiguous buffers, page i of the output = page
 * page_ids[i] of the pool, bytes verbatim.
 *
 *   k_pool_layer, v_pool_layer  dev  num_pages * page_bytes each
 *   page_ids                    dev  [n] int32 in [0, num_pages); duplicates allowed
 *   k_out, v_out                dev  n * page_bytes each
 *
 * page_bytes must be a multiple of 16 and every pointer 16-byte aligned.
 * n == 0 is MC_OK and enqueues nothing.
 */
mc_status mc_kv_pack_layer(const void* k_pool_layer, const void* v_pool_layer, int64_t num_pages,
                           int64_t page_bytes, const int32_t* page_ids, int64_t n, void* k_out,
                           void* v_out, void* hip_stream);

/*
 * Load path of layer-wise prefill (Section 5.2; Section 3 step 1): scatter
 * contiguous buffers of n pages into the listed pages of one layer's pools,
 * page page_ids[i] of the pool = page i of the input.  Pages not listed keep
 * their bytes.  page_ids must be unique (duplicates: undefined which copy wins).
 */
mc_status mc_kv_unpack_layer(const void* k_in, const void* v_in, int64_t num_pages,
                             int64_t page_bytes, const int32_t* page_ids, int64_t n,
                             void* k_pool_layer, void* v_pool_layer, void* hip_stream);

/*
 * Debugging aid for the rule above that ids in device memory are not range-checked by the calls
 * that use them (an id outside the pool makes those kernels read or write outside it): counts
 * the ids of a list that lie outside [0, num_pages).
 *
 *   page_ids  dev  int32 [n]: a pack / unpack list, or the used part of a block-table row
 *                  (ceil((P_r + C_r) / page_size) entries; entries past it are never read)
 *   report    dev  int32 [2]: report[0] = how many ids are outside the range,
 *                  report[1] = position of the first of them, n if there is none
 *
 * Enqueued like everything else: read `report` after the stream has passed the call.  n == 0
 * enqueues nothing and leaves `report` alone; n > INT32_MAX is MC_ERR_RANGE.
 */
mc_status mc_kv_check_page_ids(const int32_t* page_ids, int64_t n, int64_t num_pages, int32_t* report,
                               void* hip_stream);

/*
 * The same two copies with the order in which the pages are taken chosen by the caller.  A
 * request's page list is the same for all layers, so it pays to compute once
 *
 *   order[r] = the position in page_ids of the r-th smallest page id (equal ids: lower position
 *              first) - what mc_kv_page_order writes -
 *
 * and hand it to every layer's pack / unpack: the scattered side of the copy then walks the pool
 * in ascending address order, which the HBM sustains at a higher rate than a random walk.  The
 * bytes moved and where they land are exactly those of mc_kv_pack_layer / mc_kv_unpack_layer;
 * `order` must be a permutation of 0 .. n-1 (not checked: entries outside that range are
 * undefined behaviour, a repeated entry leaves pages uncopied), or NULL for list order.
 *
 *   order  dev  int32 [n]
 * mc_kv_page_order costs O(n^2 / threads) and rejects n > 2^20 with MC_ERR_RANGE.
 */
mc_status mc_kv_page_order(const int32_t* page_ids, int64_t n, int32_t* order, void* hip_stream);
mc_status mc_kv_pack_layer_ordered(const void* k_pool_layer, const void* v_pool_layer, int64_t num_pages,
                                   int64_t page_bytes, const int32_t* page_ids, const int32_t* order,
                                   int64_t n, void* k_out, void* v_out, void* hip_stream);
mc_status mc_kv_unpack_layer_ordered(const void* k_in, const void* v_in, int64_t num_pages,
                                     int64_t page_bytes, const int32_t* page_ids, const int32_t* order,
                                     int64_t n, void* k_pool_layer, void* v_pool_layer, void* hip_stream);

/*
 * Layer-wise prefill against the CPU-DRAM KVCache pool (Section 5.2: a layer's KVCache is loaded
 * before its attention and stored after it, asynchronously; Section 3 steps 1 and 3: the prefix
 * comes from, and the new KVCache goes back to, host memory).  One layer, one direction, all on
 * `hip_stream`:
 *
 *   load:  k_host/v_host (n packed pages each) -> k_stage/v_stage -> pages page_ids[i] of the pools
 *          = two host-to-device copies, then mc_kv_unpack_layer
 *   store: pages page_ids[i] of the pools -> k_stage/v_stage -> k_host/v_host
 *          = mc_kv_pack_layer, then two device-to-host copies
 *
 *   k_host, v_host    host  n * page_bytes each.  For the copies to be asynchronous the memory
 *                           must be pinned (hipHostMalloc); pageable memory works but blocks.
 *                           The caller keeps it valid until the stream has passed the call.
 *   k_stage, v_stage  dev   n * page_bytes each, the packed form in HBM
 *   the rest as in mc_kv_unpack_layer / mc_kv_pack_layer, same status codes.
 */
mc_status mc_kv_load_layer(const void* k_host, const void* v_host, void* k_stage, void* v_stage,
                           int64_t num_pages, int64_t page_bytes, const int32_t* page_ids, int64_t n,
                           void* k_pool_layer, void* v_pool_layer, void* hip_stream);
mc_status mc_kv_store_layer(const void* k_pool_layer, const void* v_pool_layer, int64_t num_pages,
                            int64_t page_bytes, const int32_t* page_ids, int64_t n, void* k_stage,
                            void* v_stage, void* k_host, void* v_host, void* hip_stream);

/*
 * Prefix block keys (Algorithm 1, PrefixHash; Figure "KVCache pool": a block's hash value is
 * determined by its own hash and by its prefix; Section 4: blocks of 512 tokens, one id per
 * block, the last block of a prompt may be partial).  The paper does not fix the hash; this one,
 * in 64-bit wrap-around arithmetic:
 *
 *   mix(x)    = x += 0x9E3779B97F4A7C15; x = (x ^ x >> 30) * 0xBF58476D1CE4E5B9;
 *               x = (x ^ x >> 27) * 0x94D049BB133111EB; return x ^ x >> 31      (splitmix64 output)
 *   digest(b) = mix( n_b + sum_{j < n_b} mix( (uint64)(uint32) token_j + (j << 32) ) ),  n_b tokens in block b
 *   key(0)    = mix( digest(0) ^ 0x243F6A8885A308D3 )
 *   key(b)    = mix( digest(b) ^ rotl64(key(b-1), 23) * 0x9E3779B97F4A7C15 )
 *
 *   tokens       dev   int32, requests back to back
 *   tok_offsets  host  [batch + 1], request r = tokens[tok_offsets[r] .. tok_offsets[r+1])
 *   keys         dev   uint64, request r's ceil(len_r / block_tokens) keys back to back in request order
 *   workspace    dev   >= mc_prefix_hash_workspace_bytes(batch), 16-byte aligned
 *
 * A request of more than 2^26 - 8 blocks is MC_ERR_RANGE; batch == 0 or no tokens at all is MC_OK and
 * enqueues nothing.
 */
size_t mc_prefix_hash_workspace_bytes(int32_t batch);
mc_status mc_prefix_hash(const int32_t* tokens, const int64_t* tok_offsets, int32_t batch, int32_t block_tokens,
                         uint64_t* keys, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Longest prefix match (Algorithm 1, FindBestPrefixMatch: a request's block keys are compared
 * one by one against each prefill instance's cache keys).
 *
 *   keys          dev   uint64, request r = keys[key_offsets[r] .. key_offsets[r+1])
 *   key_offsets   host  [batch + 1]
 *   cache_keys    dev   uint64, instance i = cache_keys[cache_offsets[i] .. cache_offsets[i+1]),
 *                       ASCENDING within an instance (not checked: undefined result otherwise)
 *   cache_offsets host  [n_inst + 1]
 *   prefix_len    dev   int32 [batch, n_inst]: number of LEADING keys of request r that instance
 *                       i holds (the first key it lacks ends the match)
 *   best_len      dev   int32 [batch]: the largest of them (0 if n_inst == 0)
 *   best_inst     dev   int32 [batch]: the lowest instance index attaining it (-1 if n_inst == 0)
 *   workspace     dev   >= mc_prefix_match_workspace_bytes(batch, n_inst), 16-byte aligned
 */
size_t mc_prefix_match_workspace_bytes(int32_t batch, int32_t n_inst);
mc_status mc_prefix_match(const uint64_t* keys, const int64_t* key_offsets, int32_t batch,
                          const uint64_t* cache_keys, const int64_t* cache_offsets, int32_t n_inst,
                          int32_t* prefix_len, int32_t* best_len, int32_t* best_inst, void* workspace,
                          size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MC_H_ */
