// Host side of libfdc: error text, the ragged cache layout and the work partitioner.
// Integer arithmetic only; no GPU is needed for anything in this file.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <new>
#include <numeric>
#include <queue>
#include <utility>

#include "fdc_internal.h"

namespace fdc {

static thread_local std::string g_error;

void set_error(const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  try {
    g_error = buf;
  } catch (...) {   // no memory even for the text: keep whatever was there
  }
}

// Min-heap of (load, worker id): the top is the least-loaded worker, ties to the lowest id.
using Load = std::pair<int64_t, int32_t>;
using LoadHeap = std::priority_queue<Load, std::vector<Load>, std::greater<Load>>;

static LoadHeap empty_workers(int W) {
  std::vector<Load> v(W);
  for (int w = 0; w < W; ++w) v[w] = Load(0, w);
  return LoadHeap(std::greater<Load>(), std::move(v));
}

template <class T>
static size_t append_aligned(std::vector<unsigned char>& img, const T* data, size_t count) {
  size_t off = (img.size() + 255) / 256 * 256;
  img.resize(off + std::max<size_t>(count * sizeof(T), 16));
  if (count) std::memcpy(img.data() + off, data, count * sizeof(T));
  return off;
}

static void worker_csr(const std::vector<std::vector<int32_t>>& lists, fdc_plan* p) {
  p->worker_ptr.assign(1, 0);
  p->worker_items.clear();
  for (const auto& l : lists) {
    p->worker_items.insert(p->worker_items.end(), l.begin(), l.end());
    p->worker_ptr.push_back((int32_t)p->worker_items.size());
  }
}

}  // namespace fdc

using namespace fdc;

extern "C" {

void fdc_last_error(char* buf, size_t n) {
  if (!buf || n == 0) return;
  std::strncpy(buf, g_error.c_str(), n - 1);
  buf[n - 1] = '\0';
}

// ------------------------------------------------------------------------------------ layout
fdc_status fdc_layout_create(int n_layers, int n_heads, int d_model, int d_head, const int32_t* rk,
                             const int32_t* rv, int max_batch, int max_seq, fdc_dtype dtype,
                             fdc_layout** out) {
  if (!out) FDC_FAIL(FDC_INVALID_ARG, "fdc_layout_create: out is NULL");
  *out = nullptr;
  if (!rk || !rv) FDC_FAIL(FDC_INVALID_ARG, "fdc_layout_create: rk/rv is NULL");
  if (n_layers <= 0 || n_heads <= 0 || d_model <= 0 || max_batch <= 0 || max_seq <= 0)
    FDC_FAIL(FDC_BAD_SHAPE, "fdc_layout_create: non-positive dimension");
  if (d_head < 16 || d_head > 128 || d_head % 16 != 0)
    FDC_FAIL(FDC_BAD_SHAPE, "fdc_layout_create: d_head %d must be a multiple of 16 in [16, 128]", d_head);
  if (d_model % 8 != 0) FDC_FAIL(FDC_BAD_SHAPE, "fdc_layout_create: d_model %d must be a multiple of 8", d_model);
  if (dtype != FDC_BF16 && dtype != FDC_F32 && dtype != FDC_FP8 && dtype != FDC_FP4)
    FDC_FAIL(FDC_UNSUPPORTED_DTYPE, "fdc_layout_create: dtype %d", (int)dtype);
  const size_t n = (size_t)n_layers * n_heads;
  for (size_t i = 0; i < n; ++i) {
    for (int32_t r : {rk[i], rv[i]})
      if (r < 16 || r > d_head || r % 16 != 0)
        FDC_FAIL(FDC_UNSUPPORTED_RANK, "fdc_layout_create: rank %d at index %zu is not a multiple of 16 in [16, %d]",
                 r, i, d_head);
  }
  return guarded("fdc_layout_create", [&]() -> fdc_status {
  std::unique_ptr<fdc_layout> holder(new fdc_layout());
  fdc_layout* lay = holder.get();
  lay->L = n_layers, lay->H = n_heads, lay->d_model = d_model, lay->d_head = d_head;
  lay->max_batch = max_batch, lay->max_seq = max_seq, lay->dtype = dtype;
  lay->elem_bits = dtype == FDC_BF16 ? 16 : (dtype == FDC_FP8 ? 8 : (dtype == FDC_FP4 ? 4 : 32));
  lay->rk.assign(rk, rk + n);
  lay->rv.assign(rv, rv + n);
  lay->koff.resize(n), lay->voff.resize(n);
  lay->koff_r.resize((size_t)n_layers * (n_heads + 1));
  lay->voff_r.resize((size_t)n_layers * (n_heads + 1));
  lay->k_elems.resize(n_layers), lay->v_elems.resize(n_layers);
  for (int l = 0; l < n_layers; ++l) {
    int32_t runk = 0, runv = 0;
    for (int h = 0; h < n_heads; ++h) {
      const size_t i = (size_t)l * n_heads + h, j = (size_t)l * (n_heads + 1) + h;
      lay->koff_r[j] = runk, lay->voff_r[j] = runv;
      lay->koff[i] = (int64_t)max_seq * runk, lay->voff[i] = (int64_t)max_seq * runv;
      runk += rk[i], runv += rv[i];
    }
    lay->koff_r[(size_t)l * (n_heads + 1) + n_heads] = runk;
    lay->voff_r[(size_t)l * (n_heads + 1) + n_heads] = runv;
    lay->k_elems[l] = (int64_t)max_batch * max_seq * runk;
    lay->v_elems[l] = (int64_t)max_batch * max_seq * runv;
  }
  *out = holder.release();
  return FDC_OK;
  });
}

fdc_status fdc_layout_create_gqa(int n_layers, int n_kv_heads, int q_per_kv, int d_model, int d_head, const int32_t* rk,
                                 const int32_t* rv, int max_batch, int max_seq, fdc_dtype dtype, fdc_layout** out) {
  if (!out) FDC_FAIL(FDC_INVALID_ARG, "fdc_layout_create_gqa: out is NULL");
  *out = nullptr;
  if (q_per_kv < 1 || q_per_kv > 16)
    FDC_FAIL(FDC_BAD_SHAPE, "fdc_layout_create_gqa: q_per_kv %d outside [1, 16]", q_per_kv);
  if (n_kv_heads > 0 && (int64_t)n_kv_heads * q_per_kv > 128)
    FDC_FAIL(FDC_BAD_SHAPE, "fdc_layout_create_gqa: more than 128 query heads");
  fdc_status st = fdc_layout_create(n_layers, n_kv_heads, d_model, d_head, rk, rv, max_batch, max_seq, dtype, out);
  if (st == FDC_OK) (*out)->G = q_per_kv;
  return st;
}

fdc_status fdc_layout_tables(const fdc_layout* lay, int64_t* koff, int64_t* voff, int32_t* koff_r,
                             int32_t* voff_r, int64_t* k_bytes, int64_t* v_bytes) {
  if (!lay) FDC_FAIL(FDC_INVALID_ARG, "fdc_layout_tables: layout is NULL");
  if (koff) std::copy(lay->koff.begin(), lay->koff.end(), koff);
  if (voff) std::copy(lay->voff.begin(), lay->voff.end(), voff);
  if (koff_r) std::copy(lay->koff_r.begin(), lay->koff_r.end(), koff_r);
  if (voff_r) std::copy(lay->voff_r.begin(), lay->voff_r.end(), voff_r);
  for (int l = 0; l < lay->L; ++l) {
    if (k_bytes) k_bytes[l] = lay->k_elems[l] * lay->elem_bits / 8;   // ranks are multiples of 16: whole bytes
    if (v_bytes) v_bytes[l] = lay->v_elems[l] * lay->elem_bits / 8;
  }
  return FDC_OK;
}

void fdc_layout_destroy(fdc_layout* lay) { delete lay; }

// ------------------------------------------------------------------------------------ rank selection
fdc_status fdc_select_ranks(int n, int d_head, const double* theta, double r, int multiple, int32_t* ranks) {
  if (!theta || !ranks) FDC_FAIL(FDC_INVALID_ARG, "fdc_select_ranks: NULL argument");
  if (n < 0 || d_head <= 0 || multiple <= 0) FDC_FAIL(FDC_BAD_SHAPE, "fdc_select_ranks: bad sizes");
  return guarded("fdc_select_ranks", [&]() -> fdc_status {
  std::vector<double> tails((size_t)d_head + 1);
  for (int h = 0; h < n; ++h) {
    const double* th = theta + (size_t)h * d_head;
    tails[d_head] = 0.0;
    for (int j = d_head - 1; j >= 0; --j) tails[j] = tails[j + 1] + th[j];
    const double bound = r * tails[0];
    int j_found = 0;
    for (int j = 0; j < d_head; ++j)
      if (tails[j] > bound) j_found = j;
    ranks[h] = (int32_t)((j_found + 1 + multiple - 1) / multiple * multiple);
  }
  return FDC_OK;
  });
}

// ------------------------------------------------------------------------------------ planner
void fdc_plan_params_default(fdc_plan_params* p) {
  if (!p) return;
  p->n_workers = 0;
  p->granule = 64;
  p->min_split = 1;
  p->split = 1;
  p->br_base = 64;
  p->br_cap = 256;
  p->cost_mode = 0;
  p->softmax_cost = 1;
}

static fdc_status check_plan_args(const char* fn, const fdc_layout* lay, int layer, int batch,
                                  const void* lens, const fdc_plan_params* pr, fdc_plan** out) {
  if (!out) FDC_FAIL(FDC_INVALID_ARG, "%s: out is NULL", fn);
  *out = nullptr;
  if (!lay || !lens || !pr) FDC_FAIL(FDC_INVALID_ARG, "%s: NULL argument", fn);
  if (layer < 0 || layer >= lay->L) FDC_FAIL(FDC_BAD_SHAPE, "%s: layer %d outside [0, %d)", fn, layer, lay->L);
  if (batch <= 0 || batch > lay->max_batch)
    FDC_FAIL(FDC_BAD_SHAPE, "%s: batch %d outside [1, %d]", fn, batch, lay->max_batch);
  if (pr->n_workers <= 0) FDC_FAIL(FDC_INVALID_ARG, "%s: n_workers must be positive", fn);
  if (pr->softmax_cost <= 0) FDC_FAIL(FDC_INVALID_ARG, "%s: softmax_cost must be positive", fn);
  return FDC_OK;
}

}  // extern "C"

// Decode planning. block_table == nullptr: the dense layout (sequence b is batch row b of the cache).
// Otherwise the cache is paged: the layout's batch rows are pages of P = lay->max_seq tokens and
// block_table[b * max_pages + i] is the page that holds tokens i*P .. of sequence b.
static fdc_status plan_decode_impl(const char* fn, const fdc_layout* lay, int layer, int batch,
                                   const int32_t* seq_len, const int32_t* block_table, int max_pages,
                                   const fdc_plan_params* pr, fdc_plan** out) {
  if (!out) FDC_FAIL(FDC_INVALID_ARG, "%s: out is NULL", fn);
  *out = nullptr;
  if (!lay || !seq_len || !pr) FDC_FAIL(FDC_INVALID_ARG, "%s: NULL argument", fn);
  if (layer < 0 || layer >= lay->L) FDC_FAIL(FDC_BAD_SHAPE, "%s: layer %d outside [0, %d)", fn, layer, lay->L);
  const bool paged = block_table != nullptr;
  if (batch <= 0 || (!paged && batch > lay->max_batch))
    FDC_FAIL(FDC_BAD_SHAPE, "%s: batch %d outside [1, %d]", fn, batch, lay->max_batch);
  if (pr->n_workers <= 0) FDC_FAIL(FDC_INVALID_ARG, "%s: n_workers must be positive", fn);
  if (pr->softmax_cost <= 0) FDC_FAIL(FDC_INVALID_ARG, "%s: softmax_cost must be positive", fn);
  if (pr->granule <= 0 || pr->min_split <= 0)
    FDC_FAIL(FDC_INVALID_ARG, "%s: granule and min_split must be positive", fn);
  const int64_t P = paged ? lay->max_seq : 0;   // page size in tokens (0: not paged)
  if (paged) {
    if (max_pages <= 0) FDC_FAIL(FDC_BAD_SHAPE, "%s: max_pages must be positive", fn);
    if (P % pr->granule != 0)
      FDC_FAIL(FDC_INVALID_ARG, "%s: the page size %d must be a multiple of the granule %d", fn, (int)P, pr->granule);
  }
  const int64_t seq_cap = paged ? P * max_pages : lay->max_seq;
  for (int b = 0; b < batch; ++b) {
    if (seq_len[b] < 0 || seq_len[b] > seq_cap)
      FDC_FAIL(FDC_BAD_SHAPE, "%s: seq_len[%d] = %d outside [0, %lld]", fn, b, seq_len[b], (long long)seq_cap);
    if (paged)
      for (int64_t i = 0; i < ceil_div(seq_len[b], P); ++i) {
        const int32_t pg = block_table[(size_t)b * max_pages + i];
        if (pg < 0 || pg >= lay->max_batch)
          FDC_FAIL(FDC_BAD_SHAPE, "%s: block_table[%d][%lld] = %d outside [0, %d)", fn, b, (long long)i, pg, lay->max_batch);
      }
  }

  const int H = lay->H, W = pr->n_workers;
  const int64_t G = pr->granule;
  const int32_t* rk = &lay->rk[(size_t)layer * H];
  const int32_t* rv = &lay->rv[(size_t)layer * H];
  std::vector<int64_t> d_sum(H);
  int64_t d_max = 0;
  for (int h = 0; h < H; ++h) d_sum[h] = (int64_t)rk[h] + rv[h] + pr->softmax_cost, d_max = std::max(d_max, d_sum[h]);
  int64_t total = 0;
  for (int b = 0; b < batch; ++b)
    for (int h = 0; h < H; ++h) total += seq_len[b] * d_sum[h];

  // chunks: every non-empty unit cut into min_split near-equal, granule-aligned parts
  struct Chunk { int32_t b, h, t0, t1; int64_t cost; };
  std::vector<Chunk> chunks;
  for (int b = 0; b < batch; ++b) {
    const int64_t S = seq_len[b];
    if (S == 0) continue;
    for (int h = 0; h < H; ++h) {
      int64_t n = std::max<int64_t>(1, std::min<int64_t>(pr->min_split, ceil_div(S, G)));
      const int64_t size = round_up(ceil_div(S, n), G);
      n = ceil_div(S, size);
      for (int64_t j = 0; j < n; ++j) {
        const int64_t t0 = j * size, t1 = std::min(S, (j + 1) * size);
        chunks.push_back({b, h, (int32_t)t0, (int32_t)t1, (t1 - t0) * d_sum[h]});
      }
    }
  }
  std::vector<int32_t> order(chunks.size());
  std::iota(order.begin(), order.end(), 0);
  std::sort(order.begin(), order.end(), [&](int32_t a, int32_t c) {
    return chunks[a].cost != chunks[c].cost ? chunks[a].cost > chunks[c].cost : a < c;
  });

  // list scheduling with the per-worker mean-load fill
  struct Piece { int32_t b, h, t0, t1, w; };
  std::vector<Piece> pieces;
  const int64_t mean = ceil_div(total, W);
  // Least-loaded worker, ties to the lowest id. Every piece has a positive cost, so a worker that has
  // been given one never ties with an untouched one: until all W have been touched the answer is the
  // next untouched worker, and only the touched ones need the heap (same order, a third of the work).
  LoadHeap heap;
  int32_t next_fresh = 0;
  pieces.reserve(chunks.size() + (size_t)W);
  for (int32_t ci : order) {
    const Chunk& c = chunks[ci];
    int64_t t0 = c.t0;
    while (t0 < c.t1) {
      Load top;
      if (next_fresh < W) {
        top = {0, next_fresh++};
      } else {
        top = heap.top();
        heap.pop();
      }
      int64_t take = c.t1 - t0;
      if (pr->split) {
        const int64_t room = mean - top.first, step = G * d_sum[c.h];
        const int64_t fit = std::max<int64_t>(1, (2 * room + step) / (2 * step)) * G;
        take = std::min(take, fit);
      }
      for (int64_t lo = t0, end = t0 + take; lo < end;) {   // one piece per page it touches
        const int64_t hi = P > 0 ? std::min(end, (lo / P + 1) * P) : end;
        pieces.push_back({c.b, c.h, (int32_t)lo, (int32_t)hi, top.second});
        lo = hi;
      }
      top.first += take * d_sum[c.h];
      heap.push(top);
      t0 += take;
    }
  }

  // tiles = pieces numbered by (unit, t0): sort packed keys (unit, t0, piece) instead of indices
  const size_t n = pieces.size();
  std::vector<std::pair<uint64_t, int32_t>> keyed(n);
  for (size_t k = 0; k < n; ++k)
    keyed[k] = {((uint64_t)((int64_t)pieces[k].b * H + pieces[k].h) << 32) | (uint32_t)pieces[k].t0, (int32_t)k};
  std::sort(keyed.begin(), keyed.end());
  std::vector<int32_t> by_unit(n), tile_of_piece(n);
  for (size_t tid = 0; tid < n; ++tid) {
    by_unit[tid] = keyed[tid].second;
    tile_of_piece[keyed[tid].second] = (int32_t)tid;
  }

  std::unique_ptr<fdc_plan> holder(new fdc_plan());
  fdc_plan* p = holder.get();
  p->kind = 0, p->layer = layer, p->batch = batch, p->H = H, p->n_workers = W, p->n_units = batch * H;
  p->G = lay->G;
  p->lay = lay, p->RK = lay->RK(layer), p->RV = lay->RV(layer), p->total_q_rows = batch;
  p->item_b.resize(n), p->item_h.resize(n), p->item_lo.resize(n), p->item_hi.resize(n), p->item_cost.resize(n);
  p->unit_item_ptr.assign((size_t)p->n_units + 1, 0);
  for (size_t tid = 0; tid < n; ++tid) {
    const Piece& pc = pieces[by_unit[tid]];
    p->item_b[tid] = pc.b, p->item_h[tid] = pc.h, p->item_lo[tid] = pc.t0, p->item_hi[tid] = pc.t1;
    p->item_cost[tid] = (int64_t)(pc.t1 - pc.t0) * d_sum[pc.h];
    p->unit_item_ptr[(size_t)pc.b * H + pc.h + 1] += 1;
  }
  p->min_items_per_unit = p->n_units > 0 ? p->unit_item_ptr[1] : 0;
  for (int u = 0; u < p->n_units; ++u) {
    p->max_items_per_unit = std::max(p->max_items_per_unit, p->unit_item_ptr[u + 1]);
    p->min_items_per_unit = std::min(p->min_items_per_unit, p->unit_item_ptr[u + 1]);
    p->unit_item_ptr[u + 1] += p->unit_item_ptr[u];
  }
  // worker lists in hand-out order (pieces are in that order): counting sort into CSR form
  p->worker_load.assign(W, 0);
  p->worker_ptr.assign((size_t)W + 1, 0);
  for (size_t k = 0; k < n; ++k) {
    p->worker_ptr[pieces[k].w + 1] += 1;
    p->worker_load[pieces[k].w] += (int64_t)(pieces[k].t1 - pieces[k].t0) * d_sum[pieces[k].h];
  }
  for (int w = 0; w < W; ++w) p->worker_ptr[w + 1] += p->worker_ptr[w];
  p->worker_items.resize(n);
  {
    std::vector<int32_t> fill(p->worker_ptr.begin(), p->worker_ptr.end() - 1);
    for (size_t k = 0; k < n; ++k) p->worker_items[fill[pieces[k].w]++] = tile_of_piece[k];
  }

  // device image
  const int64_t* koff = &lay->koff[(size_t)layer * H];
  const int64_t* voff = &lay->voff[(size_t)layer * H];
  const int32_t* koff_r = &lay->koff_r[(size_t)layer * (H + 1)];
  const int32_t* voff_r = &lay->voff_r[(size_t)layer * (H + 1)];
  std::vector<DecTile> tiles(n);
  for (size_t tid = 0; tid < n; ++tid) {
    const int b = p->item_b[tid], h = p->item_h[tid];
    const int u = b * H + h;
    DecTile& t = tiles[tid];
    std::memset(&t, 0, sizeof(t));
    // cache row of the tile's first token: the sequence's own batch row, or the page that holds it
    const int64_t lo = p->item_lo[tid];
    const int64_t row = paged ? block_table[(size_t)b * max_pages + lo / P] : b;
    const int64_t in_row = paged ? lo % P : lo;
    t.k_elem = row * lay->max_seq * p->RK + koff[h] + in_row * rk[h];
    t.v_elem = row * lay->max_seq * p->RV + voff[h] + in_row * rv[h];
    t.len = p->item_hi[tid] - p->item_lo[tid];
    // with g query heads per unit the query-side tensors are g times as wide and the partial
    // slots of a unit hold its tiles once per query head: slot = g * first + j * n_u + i
    const int g = p->G, n_u = p->unit_item_ptr[u + 1] - p->unit_item_ptr[u];
    t.q_elem = g * (b * p->RK + koff_r[h]);
    t.o_elem = g * (b * p->RV + voff_r[h]);
    t.rk_rv = rk[h] | (rv[h] << 16);
    t.g = g;
    t.slot_stride = n_u;
    t.slot = n_u == 1 ? -1 : g * p->unit_item_ptr[u] + ((int32_t)tid - p->unit_item_ptr[u]);
    t.b_end = b | (p->item_hi[tid] == seq_len[b] ? (int32_t)0x80000000 : 0);
  }
  p->n_merge_units = p->n_units * p->G;
  std::vector<DecUnit> units(p->n_merge_units);
  for (int u = 0; u < p->n_units; ++u) {
    const int b = u / H, h = u % H, g = p->G;
    const int n_u = p->unit_item_ptr[u + 1] - p->unit_item_ptr[u];
    for (int j = 0; j < g; ++j) {
      const int first = g * p->unit_item_ptr[u] + j * n_u;
      units[(size_t)u * g + j] = {first, first + n_u, g * (b * p->RV + voff_r[h]) + j * rv[h], rv[h]};
    }
  }
  // device image: tiles in worker (hand-out) order, merge records, one header per worker; built in
  // place (one allocation, no intermediate copies)
  auto region = [&](size_t bytes) {
    const size_t off = (p->image.size() + 255) / 256 * 256;
    p->image.resize(off + std::max<size_t>(bytes, 16));
    return off;
  };
  p->image.reserve(n * sizeof(DecTile) + units.size() * sizeof(DecUnit) + (size_t)W * sizeof(DecWorker) + 1024);
  p->off_items = region(n * sizeof(DecTile));
  p->off_units = region(units.size() * sizeof(DecUnit));
  p->off_worker_ptr = region((size_t)W * sizeof(DecWorker));
  p->off_worker_items = p->off_worker_ptr;
  p->off_lens = region((size_t)batch * sizeof(int32_t));
  std::memcpy(p->image.data() + p->off_lens, seq_len, (size_t)batch * sizeof(int32_t));
  DecTile* wtiles = reinterpret_cast<DecTile*>(p->image.data() + p->off_items);
  for (size_t i = 0; i < n; ++i) wtiles[i] = tiles[p->worker_items[i]];
  if (!units.empty()) std::memcpy(p->image.data() + p->off_units, units.data(), units.size() * sizeof(DecUnit));
  DecWorker* heads = reinterpret_cast<DecWorker*>(p->image.data() + p->off_worker_ptr);
  // Launch slot of each worker. The tile kernels run four workers per workgroup and the hardware deals
  // workgroups to the eight XCDs in turn (workgroup i -> XCD i % 8). Measured on MI355X, the even XCDs stream
  // 5 to 10 % faster than the odd ones whatever the workload, and what list scheduling leaves between
  // workers (whole granules: a few percent of the mean) is of that size. So the heavier half of the workers
  // takes the slots of the even XCDs. In load order inside each half, a compute unit's four workgroups
  // (32 workgroups of an XCD apart) come from the four quarters of it. The schedule itself is untouched.
  // (Grouped queries keep the plain order: the same ordering made that kernel 2.5 % slower, its time per tile
  // follows the planner's cost less closely.)
  std::vector<int> slot_of(W);
  for (int w = 0; w < W; ++w) slot_of[w] = w;
  if (p->G == 1 && W % (2 * kXcds * kWorkersPerGroup) == 0) {
    std::vector<int> by_load(W);
    for (int w = 0; w < W; ++w) by_load[w] = w;
    std::stable_sort(by_load.begin(), by_load.end(),
                     [&](int a, int b) { return p->worker_load[a] > p->worker_load[b]; });
    int next[2] = {0, W / 2};   // index into by_load of the next worker of the heavy / light half
    for (int s = 0; s < W; ++s) slot_of[by_load[next[((s / kWorkersPerGroup) % kXcds) % 2]++]] = s;
  }
  for (int w = 0; w < W; ++w) {
    DecWorker& hd = heads[slot_of[w]];
    hd.begin = p->worker_ptr[w];
    hd.count = p->worker_ptr[w + 1] - p->worker_ptr[w];
    if (hd.count > 0) hd.first = wtiles[hd.begin];
  }
  p->off_partials = (p->image.size() + 255) / 256 * 256;
  p->partial_bytes = std::max<size_t>(n * p->G, 1) * kPartialStride * sizeof(float);
  p->workspace_bytes = p->off_partials + p->partial_bytes;
  *out = holder.release();
  return FDC_OK;
}

extern "C" {

fdc_status fdc_plan_decode(const fdc_layout* lay, int layer, int batch, const int32_t* seq_len,
                           const fdc_plan_params* pr, fdc_plan** out) {
  return guarded("fdc_plan_decode", [&] { return plan_decode_impl("fdc_plan_decode", lay, layer, batch, seq_len, nullptr, 0, pr, out); });
}

fdc_status fdc_plan_decode_paged(const fdc_layout* lay, int layer, int batch, const int32_t* seq_len,
                                 const int32_t* block_table, int max_pages, const fdc_plan_params* pr,
                                 fdc_plan** out) {
  if (!block_table) {
    if (out) *out = nullptr;
    FDC_FAIL(FDC_INVALID_ARG, "fdc_plan_decode_paged: block_table is NULL");
  }
  return guarded("fdc_plan_decode_paged", [&] {
    return plan_decode_impl("fdc_plan_decode_paged", lay, layer, batch, seq_len, block_table, max_pages, pr, out);
  });
}

}  // extern "C"

// Prefill planning. block_table == nullptr: the dense layout. Otherwise the cache is paged as in
// plan_decode_impl; the schedule does not depend on it (a task is a block of query rows), only the
// addresses the kernel derives per staged block do.
static fdc_status plan_prefill_impl(const char* fn, const fdc_layout* lay, int layer, int batch,
                                    const int32_t* q_len, const int32_t* kv_len, const int32_t* block_table,
                                    int max_pages, const fdc_plan_params* pr, fdc_plan** out) {
  if (!out) FDC_FAIL(FDC_INVALID_ARG, "%s: out is NULL", fn);
  *out = nullptr;
  if (!lay || !q_len || !kv_len || !pr) FDC_FAIL(FDC_INVALID_ARG, "%s: NULL argument", fn);
  if (layer < 0 || layer >= lay->L) FDC_FAIL(FDC_BAD_SHAPE, "%s: layer %d outside [0, %d)", fn, layer, lay->L);
  const bool paged = block_table != nullptr;
  if (batch <= 0 || (!paged && batch > lay->max_batch))
    FDC_FAIL(FDC_BAD_SHAPE, "%s: batch %d outside [1, %d]", fn, batch, lay->max_batch);
  if (pr->n_workers <= 0) FDC_FAIL(FDC_INVALID_ARG, "%s: n_workers must be positive", fn);
  if (pr->softmax_cost <= 0) FDC_FAIL(FDC_INVALID_ARG, "%s: softmax_cost must be positive", fn);
  if (pr->br_base <= 0 || pr->br_cap < 16 || pr->br_cap % 16 != 0)
    FDC_FAIL(FDC_INVALID_ARG, "%s: br_base must be positive and br_cap a positive multiple of 16", fn);
  if (pr->cost_mode != 0 && pr->cost_mode != 1) FDC_FAIL(FDC_INVALID_ARG, "%s: cost_mode %d", fn, pr->cost_mode);
  const int64_t P = paged ? lay->max_seq : 0;
  if (paged) {
    if (max_pages <= 0) FDC_FAIL(FDC_BAD_SHAPE, "%s: max_pages must be positive", fn);
    if (P % kPrefillBlockTokens != 0)
      FDC_FAIL(FDC_INVALID_ARG, "%s: the page size %d must be a multiple of %d tokens", fn, (int)P, kPrefillBlockTokens);
  }
  const int64_t seq_cap = paged ? P * max_pages : lay->max_seq;
  for (int b = 0; b < batch; ++b) {
    if (q_len[b] < 0 || kv_len[b] < q_len[b] || kv_len[b] > seq_cap)
      FDC_FAIL(FDC_BAD_SHAPE, "%s: need 0 <= q_len[%d]=%d <= kv_len=%d <= %lld", fn, b, q_len[b], kv_len[b],
               (long long)seq_cap);
    if (paged)
      for (int64_t i = 0; i * P < kv_len[b]; ++i) {
        const int32_t pg = block_table[(size_t)b * max_pages + i];
        if (pg < 0 || pg >= lay->max_batch)
          FDC_FAIL(FDC_BAD_SHAPE, "%s: block_table[%d][%lld] = %d outside [0, %d)", fn, b, (long long)i, pg,
                   lay->max_batch);
      }
  }

  // With grouped queries the planner's heads are the QUERY heads: query head hq has the ranks and
  // the cache blocks of key/value head hq / g and its own columns in q_lat and o_lat.
  const int g = lay->G, Hkv = lay->H, H = Hkv * g, W = pr->n_workers;
  std::vector<int32_t> rk(H), rv(H);
  for (int h = 0; h < H; ++h) rk[h] = lay->rk[(size_t)layer * Hkv + h / g], rv[h] = lay->rv[(size_t)layer * Hkv + h / g];
  std::vector<int64_t> d_sum(H);
  int64_t d_max = 0;
  for (int h = 0; h < H; ++h) d_sum[h] = (int64_t)rk[h] + rv[h] + pr->softmax_cost, d_max = std::max(d_max, d_sum[h]);

  std::unique_ptr<fdc_plan> holder(new fdc_plan());
  fdc_plan* p = holder.get();
  p->kind = 1, p->layer = layer, p->batch = batch, p->H = H, p->n_workers = W, p->n_units = batch * H;
  p->G = g;
  p->lay = lay, p->RK = lay->RK(layer), p->RV = lay->RV(layer);
  p->br.resize(H);
  for (int h = 0; h < H; ++h)
    p->br[h] = (int32_t)std::min<int64_t>(pr->br_cap, round_up(ceil_div((int64_t)pr->br_base * d_max, d_sum[h]), 16));

  struct Task { int32_t b, h, q0, q1; };
  std::vector<Task> tasks;
  for (int b = 0; b < batch; ++b)
    for (int h = 0; h < H; ++h)
      for (int32_t q0 = 0; q0 < q_len[b]; q0 += p->br[h]) tasks.push_back({b, h, q0, std::min(q_len[b], q0 + p->br[h])});

  auto cost_of = [&](const Task& t) -> int64_t {
    const int64_t rows = t.q1 - t.q0;
    if (pr->cost_mode == 0) return rows * kv_len[t.b] * d_sum[t.h];
    // sum over rows i in [q0, q1) of (kv_len - q_len + i + 1)
    const int64_t first = (int64_t)kv_len[t.b] - q_len[t.b] + t.q0 + 1, last = (int64_t)kv_len[t.b] - q_len[t.b] + t.q1;
    return (first + last) * rows / 2 * d_sum[t.h];
  };

  std::vector<std::vector<int32_t>> lists(W);
  p->worker_load.assign(W, 0);
  if (pr->cost_mode == 1) {
    std::vector<int64_t> cost(tasks.size());
    for (size_t i = 0; i < tasks.size(); ++i) cost[i] = cost_of(tasks[i]);
    std::vector<int32_t> order(tasks.size());
    std::iota(order.begin(), order.end(), 0);
    std::sort(order.begin(), order.end(),
              [&](int32_t a, int32_t c) { return cost[a] != cost[c] ? cost[a] > cost[c] : a < c; });
    LoadHeap heap = empty_workers(W);
    for (int32_t i : order) {
      Load top = heap.top();
      heap.pop();
      lists[top.second].push_back(i);
      top.first += cost[i];
      p->worker_load[top.second] += cost[i];
      heap.push(top);
    }
  } else {
    const size_t n_tasks = tasks.size(), n_last = n_tasks % W, full = n_tasks - n_last;
    for (size_t i = 0; i < full; ++i) {
      lists[i % W].push_back((int32_t)i);
      p->worker_load[i % W] += cost_of(tasks[i]);
    }
    if (n_last > 0) {
      int64_t sum = 0;
      for (size_t i = full; i < n_tasks; ++i) sum += (int64_t)(tasks[i].q1 - tasks[i].q0) * d_sum[tasks[i].h];
      const int64_t wl = ceil_div(sum, W);
      std::vector<Task> resplit;
      for (size_t i = full; i < n_tasks; ++i) {
        const Task& t = tasks[i];
        const int32_t nb = (int32_t)std::max<int64_t>(16, wl / d_sum[t.h] / 16 * 16);
        for (int32_t s = t.q0; s < t.q1; s += nb) resplit.push_back({t.b, t.h, s, std::min(t.q1, s + nb)});
      }
      tasks.resize(full);
      tasks.insert(tasks.end(), resplit.begin(), resplit.end());
      LoadHeap heap = empty_workers(W);
      for (size_t j = 0; j < resplit.size(); ++j) {
        Load top = heap.top();
        heap.pop();
        const int64_t c = cost_of(resplit[j]);
        lists[top.second].push_back((int32_t)(full + j));
        top.first += c;
        p->worker_load[top.second] += c;
        heap.push(top);
      }
    }
  }
  const size_t n = tasks.size();
  p->item_b.resize(n), p->item_h.resize(n), p->item_lo.resize(n), p->item_hi.resize(n), p->item_cost.resize(n);
  for (size_t i = 0; i < n; ++i) {
    p->item_b[i] = tasks[i].b, p->item_h[i] = tasks[i].h, p->item_lo[i] = tasks[i].q0, p->item_hi[i] = tasks[i].q1;
    p->item_cost[i] = cost_of(tasks[i]);
  }
  worker_csr(lists, p);

  // device image
  const int64_t* koff = &lay->koff[(size_t)layer * Hkv];
  const int64_t* voff = &lay->voff[(size_t)layer * Hkv];
  const int32_t* koff_r = &lay->koff_r[(size_t)layer * (Hkv + 1)];
  const int32_t* voff_r = &lay->voff_r[(size_t)layer * (Hkv + 1)];
  std::vector<int64_t> row0(batch + 1, 0);
  for (int b = 0; b < batch; ++b) row0[b + 1] = row0[b] + q_len[b];
  p->total_q_rows = row0[batch];
  std::vector<PreTask> pt(n);
  for (size_t i = 0; i < n; ++i) {
    const Task& t = tasks[i];
    PreTask& d = pt[i];
    std::memset(&d, 0, sizeof(d));
    const int hk = t.h / g, j = t.h % g;
    d.k_elem = (paged ? 0 : (int64_t)t.b * lay->max_seq * p->RK) + koff[hk];
    d.v_elem = (paged ? 0 : (int64_t)t.b * lay->max_seq * p->RV) + voff[hk];
    d.page_tokens = (int32_t)P, d.page_first = paged ? t.b * max_pages : 0;
    d.q_elem = (row0[t.b] + t.q0) * g * p->RK + g * koff_r[hk] + j * rk[t.h];
    d.o_elem = (row0[t.b] + t.q0) * g * p->RV + g * voff_r[hk] + j * rv[t.h];
    d.rows = t.q1 - t.q0;
    d.pos0 = kv_len[t.b] - q_len[t.b] + t.q0;
    d.kv_len = kv_len[t.b];
    d.rk_rv = rk[t.h] | (rv[t.h] << 16);
    d.ldq = g * p->RK, d.ldo = g * p->RV;
  }
  p->off_items = append_aligned(p->image, pt.data(), pt.size());
  p->off_units = p->off_items;
  p->off_worker_ptr = append_aligned(p->image, p->worker_ptr.data(), p->worker_ptr.size());
  p->off_worker_items = append_aligned(p->image, p->worker_items.data(), p->worker_items.size());
  if (paged) p->off_pages = append_aligned(p->image, block_table, (size_t)batch * max_pages);
  p->off_partials = (p->image.size() + 255) / 256 * 256;
  p->partial_bytes = 0;
  p->workspace_bytes = p->off_partials + 256;
  *out = holder.release();
  return FDC_OK;
}

extern "C" {

fdc_status fdc_plan_prefill(const fdc_layout* lay, int layer, int batch, const int32_t* q_len,
                            const int32_t* kv_len, const fdc_plan_params* pr, fdc_plan** out) {
  return guarded("fdc_plan_prefill", [&] { return plan_prefill_impl("fdc_plan_prefill", lay, layer, batch, q_len, kv_len, nullptr, 0, pr, out); });
}

fdc_status fdc_plan_prefill_paged(const fdc_layout* lay, int layer, int batch, const int32_t* q_len,
                                  const int32_t* kv_len, const int32_t* block_table, int max_pages,
                                  const fdc_plan_params* pr, fdc_plan** out) {
  if (!block_table) {
    if (out) *out = nullptr;
    FDC_FAIL(FDC_INVALID_ARG, "fdc_plan_prefill_paged: block_table is NULL");
  }
  return guarded("fdc_plan_prefill_paged", [&] {
    return plan_prefill_impl("fdc_plan_prefill_paged", lay, layer, batch, q_len, kv_len, block_table, max_pages, pr, out);
  });
}

fdc_status fdc_plan_export(const fdc_plan* p, fdc_plan_tables* o) {
  if (!p || !o) FDC_FAIL(FDC_INVALID_ARG, "fdc_plan_export: NULL argument");
  if (p->on_device && !p->downloaded)
    FDC_FAIL(FDC_INVALID_ARG, "fdc_plan_export: the plan's tables are on the device; call fdc_plan_download first");
  o->kind = p->kind;
  o->n_items = (int32_t)p->item_b.size();
  o->n_workers = p->n_workers;
  o->n_units = p->n_units;
  o->item_b = p->item_b.data(), o->item_h = p->item_h.data();
  o->item_lo = p->item_lo.data(), o->item_hi = p->item_hi.data();
  o->item_cost = p->item_cost.data();
  o->unit_item_ptr = p->kind == 0 ? p->unit_item_ptr.data() : nullptr;
  o->worker_ptr = p->worker_ptr.data(), o->worker_items = p->worker_items.data();
  o->worker_load = p->worker_load.data();
  o->br = p->kind == 1 ? p->br.data() : nullptr;
  return FDC_OK;
}

size_t fdc_plan_workspace_bytes(const fdc_plan* p) { return p ? p->workspace_bytes : 0; }

void fdc_plan_destroy(fdc_plan* p) { delete p; }

}  // extern "C"
