/*
 * libfdc - attention computed directly on a low-rank ("latent") KV cache with a
 * different kept rank per (layer, head), for AMD MI355X (gfx950).
 *
 * Method: FDC, "Fast KV Dimensionality Compression for Efficient LLM Inference"
 * (arXiv 2408.04107). Per head the key/value projection weight is factorised
 * W ~= A.B (Section 2); the cache stores the latent rows x.A, the query is
 * moved into latent space (q.B_k^T), attention runs on the latent tensors
 * without decompression (Section 5, steps 4-7) and the per-head work, which is
 * uneven because the kept ranks differ, is balanced by a scheduler
 * (Section 5.3).
 *
 * Conventions
 *  - Every function returns fdc_status (0 = OK, negative = error) and never
 *    throws or aborts. fdc_last_error() returns a thread-local description.
 *  - "device" pointers are HIP device memory owned by the caller; "host"
 *    pointers are ordinary host memory. The library never allocates or frees
 *    device memory. Device work is enqueued on the caller's stream (a
 *    hipStream_t passed as void*; NULL = the null stream) and the call returns
 *    without synchronising.
 *  - Kept ranks are multiples of 16 in [16, d_head] (Section 6.1,
 *    implementation: widths rounded up to 16, zero padded); anything else is
 *    FDC_UNSUPPORTED_RANK. Device pointers must be 16-byte aligned
 *    (FDC_BAD_ALIGNMENT).
 *  - dtype of a layout: FDC_BF16 = caches, activations and weights are bf16,
 *    sums are fp32; FDC_F32 = everything fp32 (small validation shapes; the
 *    prefill kernel does not support it); FDC_FP8 = the K'/V' caches hold OCP
 *    E4M3 codes (one byte per element: round to nearest even, values beyond
 *    +-448 saturate), everything else is as in a bf16 layout. No scales are
 *    stored: per-head scales fold into the factors (A divided, B_k and
 *    B_v.W_o multiplied by them), so attention works on the decoded code
 *    values (the paper combines its compression with cache quantisation in
 *    Section 6.2 and fixes no format: a reading). Every call takes FDC_FP8
 *    layouts. FDC_FP4 = the caches hold OCP E2M1 codes (the 4-bit element type of
 *    the Microscaling formats: +-{0, 0.5, 1, 1.5, 2, 3, 4, 6}; round to nearest,
 *    ties to the even mantissa, saturating at +-6), two per byte: the element
 *    with the even column index in bits 3..0, its right neighbour in bits 7..4;
 *    a buffer holds elems / 2 bytes and element offsets are halved to address it.
 *    As for FDC_FP8 no scales are stored; here a scale per (head, latent column)
 *    folds into the factors. Supported by fdc_project_latent_kv,
 *    fdc_project_and_absorb_query, fdc_rope_compress_keys,
 *    fdc_latent_attn_decode(_at, _static) and fdc_latent_attn_prefill. Grouped
 *    decode attention streams a tile once for the whole group over FDC_BF16 and
 *    FDC_FP8 caches; over FDC_FP4 and FDC_F32 caches it runs the multi-head
 *    kernel once per query head of the group (same results, g times the cache
 *    traffic).
 *  - fdc_layout and fdc_plan are host objects, immutable after creation
 *    (except that fdc_plan_download fills in the host tables of a plan whose
 *    schedule was computed on the device), destroyed by the matching call.
 */
#ifndef FDC_H_
#define FDC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FDC_OK = 0,
  FDC_INVALID_ARG = -1,
  FDC_BAD_SHAPE = -2,
  FDC_BAD_ALIGNMENT = -3,
  FDC_WORKSPACE_TOO_SMALL = -4,
  FDC_UNSUPPORTED_RANK = -5,
  FDC_HIP_ERROR = -6,
  FDC_UNSUPPORTED_DTYPE = -7
} fdc_status;

typedef enum { FDC_BF16 = 0, FDC_F32 = 1, FDC_FP8 = 2, FDC_FP4 = 3 } fdc_dtype;

typedef struct fdc_layout fdc_layout;
typedef struct fdc_plan fdc_plan;

/* Copies the calling thread's last error text into buf (NUL terminated, at most n bytes). */
void fdc_last_error(char* buf, size_t n);

/* ------------------------------------------------------------------------------------------
 * Ragged latent-KV cache layout.
 *
 * The cache keeps, per layer and per head, the compressed K' (s x k) and V' instead of K and V
 * (Section 2), with k chosen per head (Section 5.2). Per layer there are two device buffers, one
 * for K' and one for V'. Unit (b, h) is a dense row-major block [max_seq, r[h]]; the blocks of
 * a sequence are concatenated over heads and sequences over b:
 *     elem(b, h, t, i) = b * max_seq * R + off[h] + t * r[h] + i
 *     off[h] = max_seq * sum_{h' < h} r[h'],   R = sum_h r[h]
 * so any token range of a unit is one contiguous span.
 *
 * rk, rv: host int32 [n_layers * n_heads], kept ranks of K' and V' (they may differ per head).
 * ------------------------------------------------------------------------------------------ */
fdc_status fdc_layout_create(int n_layers, int n_heads, int d_model, int d_head,
                             const int32_t* rk, const int32_t* rv, int max_batch, int max_seq,
                             fdc_dtype dtype, fdc_layout** out);

/* Grouped-query layout (Section 5.1, GQA paragraph): n_kv_heads key/value heads, each shared by
 * q_per_kv consecutive query heads (query head hq uses key/value head hq / q_per_kv); 1 <= q_per_kv
 * <= 16 and n_kv_heads * q_per_kv <= 128. The cache, rk, rv and every table above are per key/value
 * head exactly as in fdc_layout_create (which is q_per_kv = 1). What changes is the width of the
 * query-side tensors, ragged by QUERY head in head order:
 *     q [T, Hq, d_head], Hq = n_kv_heads * q_per_kv
 *     q_lat [T, g*RK]: query head hq at columns g*koff_r[h] + j*rk[h] .. + rk[h]   (h = hq / g, j = hq % g)
 *     o_lat [T, g*RV]: the same with voff_r, rv
 *     Wo_t [d_model, Hq*d_head], Mt [d_model, g*RV]   (M_hq = B_v^h . W_o^hq)
 * Bk, Bv, R_t, A_cat_t stay per key/value head. fdc_latent_attn_decode reads K', V' of a head once for
 * its whole query group; prefill plans one task list per query head (item_h is the query head).
 * Grouped decode attention needs a BF16 layout. */
fdc_status fdc_layout_create_gqa(int n_layers, int n_kv_heads, int q_per_kv, int d_model, int d_head,
                                 const int32_t* rk, const int32_t* rv, int max_batch, int max_seq,
                                 fdc_dtype dtype, fdc_layout** out);

/* Writes the offset tables to host arrays (any pointer may be NULL to skip it):
 *   koff, voff  int64 [L*H]      element offset of unit (0, h) inside the layer's buffer
 *   koff_r, voff_r int32 [L*(H+1)] prefix sums of the ranks (column offsets in [T, RK] tensors)
 *   k_bytes, v_bytes int64 [L]   size of the layer's K' / V' buffer in bytes                  */
fdc_status fdc_layout_tables(const fdc_layout* lay, int64_t* koff, int64_t* voff, int32_t* koff_r,
                             int32_t* voff_r, int64_t* k_bytes, int64_t* v_bytes);

void fdc_layout_destroy(fdc_layout* lay);

/* Per-head kept rank from singular values and the shared removal rate r (Section 5.2, Eq. 1):
 * the last kept dimension j is the largest index with sum_{i >= j} theta_i > r * sum_i theta_i (the
 * removed tail carries at most a fraction r of the singular-value mass); the kept rank is j + 1,
 * rounded up to `multiple` (16 for the kernels, Section 6.1). Host arrays: theta double [n, d_head],
 * each row in descending order; ranks int32 [n]. Tails are accumulated in double from the last
 * dimension backwards, so the decision is reproducible. r >= 1 keeps one dimension. */
fdc_status fdc_select_ranks(int n, int d_head, const double* theta, double r, int multiple, int32_t* ranks);

/* ------------------------------------------------------------------------------------------
 * Work partitioner (Section 5.3). Host side, integer arithmetic only, deterministic.
 *
 * decode:  task cost = s_kv * d_sum, d_sum = rk + rv + 1. Tasks are sorted by descending cost
 *          (ties: lower id first) and handed one at a time to the worker with the smallest
 *          accumulated cost (ties: lowest worker). Extension (split != 0): every unit is first cut
 *          into min_split near-equal chunks on multiples of `granule` tokens; a worker is filled
 *          only up to the mean load, a chunk that does not fit is cut at the nearest granule and
 *          its remainder goes to the next least-loaded worker. The partial softmax states of a
 *          split unit are merged exactly by fdc_latent_attn_decode.
 * prefill: head i uses row block B_r_i = round_up_16(ceil(br_base * d_sum_max / d_sum_i)), capped
 *          at br_cap. cost_mode 0 (paper): task cost rows * s_kv * d_sum; full rounds of
 *          n_workers tasks are dealt round-robin in task order; the tasks of an incomplete last
 *          round are re-split with row block max(16, floor_16(wl / d_sum_i)),
 *          wl = ceil(sum_last rows_i * d_sum_i / n_workers), and handed in order to the
 *          least-loaded worker. cost_mode 1 (causal): task cost counts only the keys a causal
 *          query row sees; all tasks are handed out in descending cost order.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int32_t n_workers; /* > 0. A worker is one wavefront (decode) or one workgroup (prefill). */
  int32_t granule;   /* decode: token granularity of cuts (default 64) */
  int32_t min_split; /* decode: minimum number of chunks per unit (default 1) */
  int32_t split;     /* decode: 1 = divisible-work extension, 0 = the paper's one task per head */
  int32_t br_base;   /* prefill: base row block (default 64) */
  int32_t br_cap;    /* prefill: largest row block (default 256) */
  int32_t cost_mode; /* prefill: 0 = paper, 1 = causal */
  int32_t softmax_cost; /* the "+ 1" of d_sum = rk + rv + 1 (default 1 = the paper's flop count); a larger
                           value weighs the per-score softmax work as that many multiply-adds */
} fdc_plan_params;

/* Fills *p with the defaults above and n_workers = 0 (the caller must set it, e.g. from
 * fdc_suggest_workers). */
void fdc_plan_params_default(fdc_plan_params* p);

/* Number of workers that are resident at once on the current HIP device for the decode
 * (kind 0), prefill (kind 1), grouped-query decode (kind 2, layouts with q_per_kv > 1), E4M3-cache
 * decode (kind 3, FDC_FP8 layouts) or E2M1-cache decode (kind 4, FDC_FP4 layouts) kernel.
 * Needs a GPU (FDC_HIP_ERROR otherwise). */
fdc_status fdc_suggest_workers(int kind, int32_t* n_workers);

/* seq_len: host int32 [batch], 0 <= seq_len[b] <= max_seq. */
fdc_status fdc_plan_decode(const fdc_layout* lay, int layer, int batch, const int32_t* seq_len,
                           const fdc_plan_params* params, fdc_plan** out);

/* Decode plan over a PAGED cache (block tables, as serving systems keep them; Section 6.1 runs on
 * one). The layout describes the pages: its batch rows are the physical pages (max_batch = number of
 * pages) and max_seq = P, the tokens per page; a page holds P tokens of one sequence in the dense
 * [head][token][component] order of the layout, so fdc_project_latent_kv / fdc_rope_compress_keys
 * write a token with tok_batch = its page and tok_pos = its offset inside the page.
 *   seq_len      host int32 [batch], 0 <= seq_len[b] <= P * max_pages (batch is not limited by the layout)
 *   block_table  host int32 [batch * max_pages]: block_table[b * max_pages + i] = page of tokens
 *                i*P .. (i+1)*P - 1 of sequence b; entries past ceil(seq_len[b] / P) are not read
 * P must be a multiple of params->granule. The schedule is that of fdc_plan_decode for the same
 * seq_len; every piece is then cut at the page boundaries it contains (item_lo / item_hi are token
 * positions in the sequence). fdc_latent_attn_decode takes the plan unchanged; q_lat and o_lat are
 * indexed by sequence. */
fdc_status fdc_plan_decode_paged(const fdc_layout* lay, int layer, int batch, const int32_t* seq_len,
                                 const int32_t* block_table, int max_pages,
                                 const fdc_plan_params* params, fdc_plan** out);

/* q_len, kv_len: host int32 [batch]; the queries of sequence b are its last q_len[b] positions,
 * q_len[b] <= kv_len[b] <= max_seq. Query rows of all sequences are stacked b-major: T = sum q_len. */
fdc_status fdc_plan_prefill(const fdc_layout* lay, int layer, int batch, const int32_t* q_len,
                            const int32_t* kv_len, const fdc_plan_params* params, fdc_plan** out);

/* Prefill plan over a PAGED cache: the layout describes the pages and block_table maps them to
 * sequences exactly as for fdc_plan_decode_paged; kv_len[b] <= P * max_pages, and P must be a
 * multiple of 128 (the kernel stages K'/V' 128 tokens at a time and a block never straddles pages).
 * The schedule is that of fdc_plan_prefill for the same lengths (tasks are blocks of query rows;
 * pages do not cut them). fdc_latent_attn_prefill takes the plan unchanged. */
fdc_status fdc_plan_prefill_paged(const fdc_layout* lay, int layer, int batch, const int32_t* q_len,
                                  const int32_t* kv_len, const int32_t* block_table, int max_pages,
                                  const fdc_plan_params* params, fdc_plan** out);

/* The decode planner as a GPU kernel (Section 6.1, implementation: the scheduling computations of
 * the decode kernel, sorting included, run on the device). For callers whose sequence lengths live
 * in device memory and who do not want a host round trip per re-plan (serving loops, captured
 * graphs). The schedule and every table are those fdc_plan_decode / fdc_plan_decode_paged would
 * produce for the same lengths, bit for bit.
 *
 * fdc_plan_decode_device (host only, no GPU work) sizes a plan for ANY lengths up to the layout's
 * capacity: max_pages = 0 for the dense cache (seq_len[b] <= max_seq), max_pages > 0 for the paged
 * cache of fdc_plan_decode_paged (seq_len[b] <= P * max_pages). Its workspace is larger than that
 * of a host plan for one set of lengths (regions are sized by an upper bound on the tile count).
 * Limits of the kernel (FDC_BAD_SHAPE beyond them; fdc_plan_decode has none): n_workers <= 8192,
 * batch <= 2048, batch * n_heads * min_split <= 8192, worker loads below 2^29.
 * Use: fdc_plan_upload once (constants), then fdc_plan_decode_run whenever the lengths change, then
 * fdc_latent_attn_decode / _decode_at with (plan, workspace) as for a host plan.
 *
 * fdc_plan_decode_run launches one workgroup per plan (1 <= n_plans <= 32: e.g. the layers of a
 * model, all for the same batch and cache shape), asynchronously on `stream`:
 *   plans, workspaces  host arrays [n_plans]; workspaces[i] is the 256-byte aligned device workspace
 *                      plans[i] was uploaded to (distinct per plan)
 *   seq_len            device int32 [batch]; values outside [0, capacity] are planned clamped
 *   block_table        device int32 [batch * max_pages] (paged plans; NULL otherwise); entries outside
 *                      the layout's pages are replaced by page 0
 * Both faults are recorded in the workspace and reported by fdc_plan_download; no kernel ever reads
 * outside the cache because of them.
 *
 * fdc_plan_download (optional; synchronises `stream`) copies the tables back so that
 * fdc_plan_export works on the plan, and returns FDC_BAD_SHAPE if the kernel recorded a fault. */
fdc_status fdc_plan_decode_device(const fdc_layout* lay, int layer, int batch, int max_pages,
                                  const fdc_plan_params* params, fdc_plan** out);
fdc_status fdc_plan_decode_run(fdc_plan* const* plans, void* const* workspaces, int n_plans,
                               const int32_t* seq_len, const int32_t* block_table, void* stream);
fdc_status fdc_plan_download(fdc_plan* plan, const void* workspace, void* stream);

/* Host view of a plan's tables (pointers stay valid until fdc_plan_destroy). An item is a decode
 * tile (lo, hi = token range) or a prefill task (lo, hi = query-row range). */
typedef struct {
  int32_t kind; /* 0 decode, 1 prefill */
  int32_t n_items;
  int32_t n_workers;
  int32_t n_units; /* batch * n_heads */
  const int32_t* item_b;
  const int32_t* item_h;
  const int32_t* item_lo;
  const int32_t* item_hi;
  const int64_t* item_cost;
  const int32_t* unit_item_ptr; /* decode: [n_units + 1], items of a unit are consecutive; prefill: NULL */
  const int32_t* worker_ptr;    /* [n_workers + 1] */
  const int32_t* worker_items;  /* [n_items], in hand-out order */
  const int64_t* worker_load;   /* [n_workers] */
  const int32_t* br;            /* prefill: [n_heads]; decode: NULL */
} fdc_plan_tables;

fdc_status fdc_plan_export(const fdc_plan* plan, fdc_plan_tables* out);

/* Device workspace a plan needs: its tables plus, for decode, one partial softmax state per tile. */
size_t fdc_plan_workspace_bytes(const fdc_plan* plan);

/* Copies the plan's tables into the device workspace (asynchronously on `stream`; the plan must
 * stay alive until the copy has completed). Must be called once before the attention call that
 * uses (plan, workspace). */
fdc_status fdc_plan_upload(const fdc_plan* plan, void* workspace, size_t workspace_bytes, void* stream);

void fdc_plan_destroy(fdc_plan* plan);

/* ------------------------------------------------------------------------------------------
 * The five hot-path calls. All pointers below are device pointers unless marked host.
 * ------------------------------------------------------------------------------------------ */

/* K'_h = x . A_k^h and V'_h = x . A_v^h for all heads (Section 2: K' = E A), written into the
 * ragged cache: row t goes to sequence tok_batch[t], position tok_pos[t].
 *   x        [T, d_model]                       layout dtype
 *   tok_batch, tok_pos  int32 [T]               0 <= tok_batch < max_batch, 0 <= tok_pos < max_seq
 *   A_cat_t  [RK + RV, d_model] row-major       row n holds the d_model weights of latent column n
 *                                               (the "out x in" order of a linear layer); rows: all K
 *                                               heads (head-major), then all V heads
 *   k_cache, v_cache    the layer's K' / V' buffers (sizes from fdc_layout_tables)
 * k_cache may be NULL: then A_cat_t holds only the RV value rows and only V' is written (post-RoPE
 * path, where K' comes from fdc_rope_compress_keys). T = 0 is a no-op.
 *   status   device int32 (4-byte aligned) or NULL. tok_batch and tok_pos are device data the host
 *            cannot check: a row whose tok_batch is outside [0, max_batch) or whose tok_pos is outside
 *            [0, max_seq) is SKIPPED by the kernel (nothing is stored for it, every other row is written
 *            as usual) and, when status is not NULL, FDC_FAULT_TOK_BATCH / FDC_FAULT_TOK_POS is OR-ed into
 *            *status. The caller clears the word and reads it when it likes; the call itself still
 *            returns FDC_OK. The other cache writers below take the same argument. */
enum { FDC_FAULT_TOK_BATCH = 1, FDC_FAULT_TOK_POS = 2 };
fdc_status fdc_project_latent_kv(const fdc_layout* lay, int layer, const void* x, int T,
                                 const int32_t* tok_batch, const int32_t* tok_pos, const void* A_cat_t,
                                 void* k_cache, void* v_cache, int32_t* status, void* stream);

/* q'_h = q_h . (B_k^h)^T per head (Section 2: Q K^T = E (W_Q B_K^T) K'^T).
 *   q      [T, H, d_head]        layout dtype
 *   Bk     [RK, d_head]          head h = rows koff_r[h] .. koff_r[h+1]
 *   q_lat  [T, RK]               q_lat_dtype (F32 for decode, BF16 for prefill) */
fdc_status fdc_absorb_query(const fdc_layout* lay, int layer, const void* q, int T, const void* Bk,
                            void* q_lat, fdc_dtype q_lat_dtype, void* stream);

/* fdc_project_latent_kv and fdc_absorb_query of the same T tokens in one call (the two products that
 * start a decode layer, Section 2; they are independent of each other). Arguments, layouts and
 * results are those of the two calls, bit for bit. With a bf16 layout and 1 <= T <= 16 both run in
 * one kernel launch; otherwise the two calls are made in turn on `stream`. */
fdc_status fdc_project_and_absorb_query(const fdc_layout* lay, int layer, const void* x, int T,
                                        const int32_t* tok_batch, const int32_t* tok_pos, const void* A_cat_t,
                                        void* k_cache, void* v_cache, const void* q, const void* Bk, void* q_lat,
                                        fdc_dtype q_lat_dtype, int32_t* status, void* stream);

/* Post-RoPE compression of Q and K (Section 5.1; steps 5 and 6 of the design overview): RoPE, then
 * the common rotation R of the head truncated to its first r_h columns, (Q_p R_p)(K_p R_p)^T ~= Q_p K_p^T.
 * Attention, planning and the V path are unchanged; K' of the cache is written by
 * fdc_rope_compress_keys instead of fdc_project_latent_kv. BF16 layouts only.
 *   q, k      [T, H, d_head]   pre-RoPE rows of every head (outputs of the model's own W_Q / W_K)
 *   tok_pos   int32 [T]        position of each row, 0 <= tok_pos < n_pos (and < max_seq for keys)
 *   tok_batch int32 [T]        sequence of each key row
 *   cos_t, sin_t  f32 [n_pos, d_head / 2]   RoPE angles; the pair (2i, 2i+1) of a row at position p is
 *                              rotated by the angle whose cosine / sine is cos_t[p, i] / sin_t[p, i]
 *   R_t       [RK, d_head]     head h = rows koff_r[h] .. koff_r[h+1]: the first rk[h] columns of R^h,
 *                              one kept direction per row (the layout of Bk)
 *   q_lat     [T, RK] (q_lat_dtype);   k_cache: the layer's K' buffer.
 *   status    as for fdc_project_latent_kv: a row whose tok_pos has no angle (outside [0, n_pos)), and a key
 *             row whose tok_batch / tok_pos lies outside the cache, is skipped (its q_lat row / cache row
 *             is left untouched) and flagged. */
fdc_status fdc_rope_absorb_query(const fdc_layout* lay, int layer, const void* q, int T, const int32_t* tok_pos,
                                 const float* cos_t, const float* sin_t, int n_pos, const void* R_t,
                                 void* q_lat, fdc_dtype q_lat_dtype, int32_t* status, void* stream);
fdc_status fdc_rope_compress_keys(const fdc_layout* lay, int layer, const void* k, int T,
                                  const int32_t* tok_batch, const int32_t* tok_pos, const float* cos_t,
                                  const float* sin_t, int n_pos, const void* R_t, void* k_cache, int32_t* status,
                                  void* stream);

/* Decode attention on the latent cache, one query per sequence (Section 5, step 7; Section 5.3
 * decode scheduling): o'_h = softmax_t(scale * <q'_h, K'_h[t]>) . V'_h over t < seq_len[b].
 *   q_lat [batch, RK] f32, o_lat [batch, RV] f32, scale > 0 and finite, normally 1/sqrt(d_head)
 *   (FDC_INVALID_ARG otherwise; the same holds for fdc_latent_attn_prefill).
 *   workspace: prepared by fdc_plan_upload for this plan. Sequences with seq_len 0 give zeros.
 * Calls that share a workspace must not overlap in time.
 * Precision: multi-head layouts keep q', the scores and the softmax weights in fp32. Grouped-query
 * layouts run both products on the matrix core: q' enters as the sum of two bf16 terms (16 bits of
 * its mantissa), the softmax weights as bf16, sums are fp32. */
fdc_status fdc_latent_attn_decode(const fdc_layout* lay, const fdc_plan* plan, const void* q_lat,
                                  const void* k_cache, const void* v_cache, float scale, void* o_lat,
                                  void* workspace, size_t workspace_bytes, void* stream);

/* The same call for a decode loop that appends a token per step without planning every step
 * (Section 5.3 schedules per step; the schedule of a plan only depends on the lengths in units of
 * the granule). Plan once with every length rounded up to a multiple of params->granule, then call
 * this with the actual lengths:
 *   seq_len  device int32 [batch], planned[b] - granule < seq_len[b] <= planned[b] (and 0 where
 *            planned[b] is 0); read by the kernel, not checked on the host
 * The tile that ends a sequence covers only the tokens below seq_len[b]; everything else is the
 * planned call. Out-of-range entries never make a kernel read past a planned tile, but the result
 * for that sequence is then meaningless. */
fdc_status fdc_latent_attn_decode_at(const fdc_layout* lay, const fdc_plan* plan, const int32_t* seq_len,
                                     const void* q_lat, const void* k_cache, const void* v_cache, float scale,
                                     void* o_lat, void* workspace, size_t workspace_bytes, void* stream);

/* fdc_latent_attn_decode for callers that cannot allocate device memory for a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc). The plan's tables and
 * the split-K partial states live in a workspace built into the library's code object:
 * FDC_STATIC_SCRATCH_BYTES of device memory per GPU, held until the process ends. The call makes no
 * hipMalloc / hipFree and needs no fdc_plan_upload: it copies the plan's tables into the built-in
 * workspace when they are not the ones already there (host -> device copy on `stream`; the plan must
 * stay alive until it has completed), then runs the kernels of fdc_latent_attn_decode. Results are
 * those of fdc_latent_attn_decode, bit for bit.
 *   plan: a host plan (fdc_plan_decode / fdc_plan_decode_paged) whose fdc_plan_workspace_bytes is at
 *         most FDC_STATIC_SCRATCH_BYTES: FDC_WORKSPACE_TOO_SMALL beyond that, FDC_INVALID_ARG for a
 *         plan of fdc_plan_decode_device (its tables are written by a kernel into the caller's workspace).
 * All calls on one GPU share the one workspace, whatever their stream or thread: calls that overlap
 * in time on a GPU race (run them on one stream, or order them with events). */
#define FDC_STATIC_SCRATCH_BYTES ((size_t)8 << 20)
fdc_status fdc_latent_attn_decode_static(const fdc_layout* lay, const fdc_plan* plan, const void* q_lat,
                                         const void* k_cache, const void* v_cache, float scale, void* o_lat,
                                         void* stream);

/* Measurement aid: when both arguments are non-NULL hipEvent_t handles, the next
 * fdc_latent_attn_decode call made by this thread attaches them to the dispatch of its tile kernel
 * (the kernel that streams the cache): `start` takes the time that kernel begins, `stop` the time
 * it ends, on that call's stream; the split-K merge runs after `stop`. The request is consumed by
 * that call, whether it succeeds or not; NULLs cancel it. */
fdc_status fdc_profile_decode_events(void* start_event, void* stop_event);

/* Prefill attention on the latent cache (Section 5, step 7; Section 5.3 prefill scheduling).
 *   q_lat [T, RK] bf16 and o_lat [T, RV] bf16, rows stacked b-major as in fdc_plan_prefill;
 *   causal != 0: query at position p sees keys t <= p. BF16 layouts only. */
fdc_status fdc_latent_attn_prefill(const fdc_layout* lay, const fdc_plan* plan, const void* q_lat,
                                   const void* k_cache, const void* v_cache, float scale, int causal,
                                   void* o_lat, void* workspace, size_t workspace_bytes, void* stream);

/* Output absorption: the latent head outputs go straight through M = B_v . W_o (the paper
 * compresses V "following Palu"; the fold is (P V') B_v W_o = (P V') (B_v W_o)).
 * Weights are stored "out x in" (contiguous along the summed index), so W_o comes as
 * Wo_t [d_model, H*d_head] and the folded matrix is kept as Mt [d_model, RV] = M^T.
 *   mode FDC_FOLD : M_h = B_v^h . W_o^h for every head; Bv [RV, d_head], Wo_t, Mt all layout dtype
 *                   (Mt fp32 in an FDC_F32 layout). o_lat, y ignored.
 *   mode FDC_APPLY: y [T, d_model] = o_lat [T, RV] . M;  o_lat_dtype / y_dtype say how they are
 *                   stored. Bv, Wo_t ignored. In a bf16 / E4M3 layout the product runs on the matrix
 *                   core with bf16 operands: an fp32 o_lat is rounded to bf16 on its way in (the
 *                   precision Mt itself has), sums are fp32. The same holds for fp32 activations of
 *                   the other projections. */
enum { FDC_FOLD = 0, FDC_APPLY = 1 };
fdc_status fdc_absorb_output(const fdc_layout* lay, int layer, int mode, const void* Bv, const void* Wo_t,
                             void* Mt, const void* o_lat, fdc_dtype o_lat_dtype, int T, void* y,
                             fdc_dtype y_dtype, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FDC_H_ */
