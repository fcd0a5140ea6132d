// The decode work partitioner as a GPU kernel (Section 6.1, implementation of the decode kernel
// enhancement: the scheduling computations, sorting included, run on the device). The schedule is
// the one of fdc_plan_decode, table for table: chunks sorted by (cost descending, id ascending),
// handed one at a time to the least-loaded worker (ties to the lowest id), a worker filled to the
// mean load with cuts at multiples of the granule (Section 5.3 plus the divisible-work extension).
//
// One workgroup plans one layer. The parts with no order between their elements (chunk costs, the
// sort, prefix sums, the tile / worker / merge records) use all 1024 threads; the hand-out itself is
// a chain (every decision depends on the loads left by the one before), so one wavefront walks it
// and uses its 64 lanes for the only wide step, the search for the least-loaded worker: the loads
// sit in LDS in 64 segments, lane s keeps the minimum of segment s and where it is, a hand-out is
// one reduction over the 64 segment minima, one LDS write and one re-scan of the segment that
// changed.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <climits>
#include <cstring>
#include <mutex>
#include <vector>

#include "fdc_internal.h"

namespace fdc {

constexpr int kPlanThreads = 1024;
constexpr int kPlanMaxChunks = 8192;    // chunk ids take 13 bits of a sort key
constexpr int kPlanMaxWorkers = 8192;   // two loads per lane in a segment re-scan
constexpr int kPlanMaxBatch = 2048;
constexpr int kPlanMaxHeads = 4096;
constexpr int kPlanMaxLayersPerLaunch = 32;
constexpr int64_t kPlanMaxLoad = (int64_t)1 << 29;   // loads and steps stay below this: 32-bit arithmetic in the chain
constexpr size_t kPlanMaxLds = 160 * 1024;

enum : int32_t {
  kPlanBadLength = 1,   // a sequence length outside [0, cap] (planned as clamped)
  kPlanOverflow = 2,    // more pieces than the bound (nothing is scheduled)
  kPlanBadPage = 4,     // a block-table entry outside the layout's pages (page 0 is used)
};

// What a device plan keeps at the start of its workspace: constants written once by fdc_plan_upload.
// The per-head tables rk, rv, koff_r, voff_r (int32 [H] each) follow the struct.
struct DevPlanConst {
  int32_t batch, H, W, granule, min_split, split, softmax_cost, g;
  int32_t row_tokens;    // tokens of a cache row (the layout's max_seq; the page size when paged)
  int32_t page_tokens;   // 0: dense cache
  int32_t max_pages, n_pages, seq_cap;
  int32_t n_max;         // most pieces the regions below hold
  int32_t RK, RV;
  int32_t n_pad;         // sort width: power of two >= the most chunks there can be
  int32_t seg_log2;      // workers per segment = 1 << seg_log2, 64 segments cover W
  int32_t n_merge_units;
  int32_t pad0;
  // byte offsets inside the workspace
  uint64_t off_header, off_items, off_units, off_workers, off_lens, off_export, off_srec, off_chunk_cnt, off_pieces;
  // byte offsets inside dynamic LDS
  uint32_t lds_keys, lds_loads, lds_wcount, lds_len, lds_cbase, lds_dsum, lds_red, lds_bytes;
};

struct DevPlanHeader {
  int32_t n_items, max_items_per_unit, status, n_chunks;
  int64_t total, mean;
};

struct DevPlanLaunch {
  unsigned char* ws[kPlanMaxLayersPerLaunch];
};

// Export tables inside the workspace (what fdc_plan_download copies back), by n_max, n_units, W.
struct ExportOffsets {
  size_t item_b, item_h, item_lo, item_hi, worker_items, unit_item_ptr, worker_ptr, worker_load, bytes;
};
__host__ __device__ inline ExportOffsets export_offsets(int64_t n_max, int64_t n_units, int64_t W) {
  ExportOffsets e;
  size_t o = 0;
  auto take = [&](size_t bytes) { const size_t at = o; o += (bytes + 15) / 16 * 16; return at; };
  e.item_b = take(n_max * 4), e.item_h = take(n_max * 4), e.item_lo = take(n_max * 4), e.item_hi = take(n_max * 4);
  e.worker_items = take(n_max * 4);
  e.unit_item_ptr = take((n_units + 1) * 4), e.worker_ptr = take((W + 1) * 4), e.worker_load = take(W * 8);
  e.bytes = o;
  return e;
}

// Chunks of a unit of S tokens: n near-equal parts whose boundaries are multiples of the granule.
__device__ __forceinline__ void chunk_shape(int32_t S, int32_t G, int32_t min_split, int32_t* n, int32_t* size) {
  if (S <= 0) {
    *n = 0, *size = G;
    return;
  }
  int32_t k = min(min_split, (S + G - 1) / G);
  k = max(k, 1);
  const int32_t sz = ((S + k - 1) / k + G - 1) / G * G;
  *n = (S + sz - 1) / sz, *size = sz;
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}

// Minimum over the wavefront, in every lane (row reduction with DPP, then the lane-row swaps).
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
  v = min(v, dpp_u32<0xB1>(v));   // quad_perm [1,0,3,2]
  v = min(v, dpp_u32<0x4E>(v));   // quad_perm [2,3,0,1]
  v = min(v, dpp_u32<0x141>(v));  // row_half_mirror
  v = min(v, dpp_u32<0x140>(v));  // row_mirror
  auto a = __builtin_amdgcn_permlane16_swap(v, v, false, false);
  v = min(a[0], a[1]);
  auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return min(b[0], b[1]);
}

// Exclusive prefix sum of data[0..n) in place (LDS), data[n] = total. part: LDS scratch [kPlanThreads].
__device__ void block_exclusive_scan(uint32_t* data, int n, uint32_t* part) {
  const int tid = threadIdx.x;
  const int per = (n + kPlanThreads - 1) / kPlanThreads;
  const int lo = min(n, tid * per), hi = min(n, lo + per);
  uint32_t s = 0;
  for (int i = lo; i < hi; ++i) s += data[i];
  part[tid] = s;
  __syncthreads();
  for (int o = 1; o < kPlanThreads; o <<= 1) {   // inclusive scan of the per-thread sums
    const uint32_t add = tid >= o ? part[tid - o] : 0;
    __syncthreads();
    part[tid] += add;
    __syncthreads();
  }
  uint32_t run = tid > 0 ? part[tid - 1] : 0;
  for (int i = lo; i < hi; ++i) {
    const uint32_t v = data[i];
    data[i] = run;
    run += v;
  }
  if (tid == kPlanThreads - 1) data[n] = part[tid];
  __syncthreads();
}

// Sequence that owns chunk ci: the last b with cbase[b] <= ci (sequences without chunks share
// their cbase with the next one, so the last such b is the one whose range holds ci).
__device__ __forceinline__ int chunk_sequence(const uint32_t* cbase, int batch, uint32_t ci) {
  int lo = 0, hi = batch - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (cbase[mid] <= ci) lo = mid; else hi = mid - 1;
  }
  return lo;
}

__global__ __launch_bounds__(kPlanThreads) void plan_decode_kernel(DevPlanLaunch launch,
                                                                   const int32_t* __restrict__ seq_len,
                                                                   const int32_t* __restrict__ block_table) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int32_t sh_status, sh_n_items, sh_max_items;
  __shared__ int64_t sh_mean;
  unsigned char* ws = launch.ws[blockIdx.x];
  const DevPlanConst c = *reinterpret_cast<const DevPlanConst*>(ws);
  const int32_t* rk = reinterpret_cast<const int32_t*>(ws + sizeof(DevPlanConst));
  const int32_t* rv = rk + c.H;
  const int32_t* koff_r = rv + c.H;
  const int32_t* voff_r = koff_r + c.H;
  const int tid = threadIdx.x, lane = tid & 63;
  const int batch = c.batch, H = c.H, W = c.W, G = c.granule;

  uint64_t* keys = reinterpret_cast<uint64_t*>(smem + c.lds_keys);
  uint32_t* chunk_base = reinterpret_cast<uint32_t*>(smem + c.lds_keys);   // after the hand-out
  uint32_t* loads = reinterpret_cast<uint32_t*>(smem + c.lds_loads);
  uint32_t* wcount = reinterpret_cast<uint32_t*>(smem + c.lds_wcount);      // then worker_ptr, in place
  int32_t* len = reinterpret_cast<int32_t*>(smem + c.lds_len);
  uint32_t* cbase = reinterpret_cast<uint32_t*>(smem + c.lds_cbase);
  uint32_t* d_sum = reinterpret_cast<uint32_t*>(smem + c.lds_dsum);
  uint32_t* red32 = reinterpret_cast<uint32_t*>(smem + c.lds_red);
  uint64_t* red64 = reinterpret_cast<uint64_t*>(smem + c.lds_red);

  DevPlanHeader* header = reinterpret_cast<DevPlanHeader*>(ws + c.off_header);
  DecTile* wtiles = reinterpret_cast<DecTile*>(ws + c.off_items);
  DecUnit* units = reinterpret_cast<DecUnit*>(ws + c.off_units);
  DecWorker* heads = reinterpret_cast<DecWorker*>(ws + c.off_workers);
  int32_t* lens_out = reinterpret_cast<int32_t*>(ws + c.off_lens);
  int4* srec = reinterpret_cast<int4*>(ws + c.off_srec);
  uint32_t* chunk_cnt = reinterpret_cast<uint32_t*>(ws + c.off_chunk_cnt);
  int4* pieces = reinterpret_cast<int4*>(ws + c.off_pieces);
  const int n_units = batch * H;
  const ExportOffsets eo = export_offsets(c.n_max, n_units, W);
  unsigned char* ex = ws + c.off_export;
  int32_t* ex_b = reinterpret_cast<int32_t*>(ex + eo.item_b);
  int32_t* ex_h = reinterpret_cast<int32_t*>(ex + eo.item_h);
  int32_t* ex_lo = reinterpret_cast<int32_t*>(ex + eo.item_lo);
  int32_t* ex_hi = reinterpret_cast<int32_t*>(ex + eo.item_hi);
  int32_t* ex_witems = reinterpret_cast<int32_t*>(ex + eo.worker_items);
  int32_t* ex_uptr = reinterpret_cast<int32_t*>(ex + eo.unit_item_ptr);
  int32_t* ex_wptr = reinterpret_cast<int32_t*>(ex + eo.worker_ptr);
  int64_t* ex_wload = reinterpret_cast<int64_t*>(ex + eo.worker_load);

  // ---- lengths, d_sum, total cost, chunks per sequence -------------------------------------------
  if (tid == 0) sh_status = 0, sh_n_items = 0, sh_max_items = 0;
  uint32_t D = 0;   // sum of d_sum over heads (every thread computes it: H is small)
  for (int h = 0; h < H; ++h) D += (uint32_t)(rk[h] + rv[h] + c.softmax_cost);
  for (int h = tid; h < H; h += kPlanThreads) d_sum[h] = (uint32_t)(rk[h] + rv[h] + c.softmax_cost);
  __syncthreads();
  uint64_t my_total = 0;
  for (int b = tid; b < batch; b += kPlanThreads) {
    int32_t S = seq_len[b];
    if (S < 0 || S > c.seq_cap) {
      atomicOr(&sh_status, kPlanBadLength);
      S = S < 0 ? 0 : c.seq_cap;
    }
    len[b] = S, lens_out[b] = S;
    int32_t n, size;
    chunk_shape(S, G, c.min_split, &n, &size);
    cbase[b] = (uint32_t)(n * H);
    my_total += (uint64_t)S * D;
  }
  red64[tid] = my_total;
  __syncthreads();
  for (int o = kPlanThreads / 2; o > 0; o >>= 1) {
    if (tid < o) red64[tid] += red64[tid + o];
    __syncthreads();
  }
  if (tid == 0) sh_mean = (int64_t)((red64[0] + (uint64_t)W - 1) / (uint64_t)W);
  const uint64_t total = red64[0];
  __syncthreads();
  block_exclusive_scan(cbase, batch, red32);
  // values that steer the hand-out loop are made wave-uniform registers explicitly
  const int n_chunks = __builtin_amdgcn_readfirstlane((int)cbase[batch]);
  const uint32_t mean = (uint32_t)__builtin_amdgcn_readfirstlane((int)sh_mean);   // < 2^29 (checked at creation)

  // ---- sort keys: cost descending, chunk id ascending ---------------------------------------------
  for (int ci = tid; ci < c.n_pad; ci += kPlanThreads) {
    uint64_t key = 0;
    if (ci < n_chunks) {
      const int b = chunk_sequence(cbase, batch, (uint32_t)ci);
      int32_t n, size;
      chunk_shape(len[b], G, c.min_split, &n, &size);
      const int r = ci - (int)cbase[b], h = r / n, j = r % n;
      const int32_t t0 = j * size, t1 = min(len[b], t0 + size);
      key = ((uint64_t)(t1 - t0) * d_sum[h]) << 13 | (uint64_t)(kPlanMaxChunks - 1 - ci);
    }
    keys[ci] = key;
  }
  __syncthreads();
  for (int k = 2; k <= c.n_pad; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int i = tid; i < c.n_pad; i += kPlanThreads) {
        const int p = i ^ j;
        if (p > i) {
          const uint64_t a = keys[i], b = keys[p];
          const bool descending = (i & k) == 0;
          if (descending ? a < b : a > b) keys[i] = b, keys[p] = a;
        }
      }
      __syncthreads();
    }
  // chunk records in hand-out order; worker state
  for (int s = tid; s < n_chunks; s += kPlanThreads) {
    const int ci = kPlanMaxChunks - 1 - (int)(keys[s] & (kPlanMaxChunks - 1));
    const int b = chunk_sequence(cbase, batch, (uint32_t)ci);
    int32_t n, size;
    chunk_shape(len[b], G, c.min_split, &n, &size);
    const int r = ci - (int)cbase[b], h = r / n, j = r % n;
    const int32_t t0 = j * size, t1 = min(len[b], t0 + size);
    srec[s] = make_int4(b | (h << 16), ci, t0, t1);
  }
  const int seg = 1 << c.seg_log2;
  for (int w = tid; w < 64 * seg; w += kPlanThreads) loads[w] = w < W ? 0u : 0xffffffffu, wcount[w] = 0;
  __syncthreads();

  // ---- the hand-out: one wavefront ------------------------------------------------------------------
  if (tid < 64) {
    const int P = __builtin_amdgcn_readfirstlane(c.page_tokens), n_max = __builtin_amdgcn_readfirstlane(c.n_max);
    const int split = __builtin_amdgcn_readfirstlane(c.split), seg_log2 = __builtin_amdgcn_readfirstlane(c.seg_log2);
    const int Gs = __builtin_amdgcn_readfirstlane(G);
    // Lane s keeps the least load of workers [s << seg_log2, (s + 1) << seg_log2) and the lowest worker
    // that has it. Every piece has a positive cost, so a worker that has been given one never ties with an
    // untouched one: until all W have been touched the least-loaded worker is the next untouched one (load
    // 0, in id order), and the segment minima are only built when that phase ends.
    uint32_t segmin = 0, segarg = 0;
    auto rescan = [&](uint32_t sg) {   // new minimum of segment sg, into lane sg
      const uint32_t base = sg << seg_log2;
      const uint32_t v0 = lane < seg ? loads[base + lane] : 0xffffffffu;
      const uint32_t v1 = lane + 64 < seg ? loads[base + 64 + lane] : 0xffffffffu;
      const uint32_t m2 = wave_min_u32(min(v0, v1));
      const uint64_t hit0 = __ballot(v0 == m2);
      const uint32_t arg = hit0 ? (uint32_t)__builtin_ctzll(hit0) : 64u + (uint32_t)__builtin_ctzll(__ballot(v1 == m2));
      if ((uint32_t)lane == sg) segmin = m2, segarg = base + arg;
    };
    // tokens a worker of load m takes of a head with this step: the nearest number of granules to
    // room / step, at least one
    auto fit_tokens = [&](uint32_t m, uint32_t step) -> int64_t {
      const int32_t num = 2 * ((int32_t)mean - (int32_t)m) + (int32_t)step;
      const int32_t fit = num >= (int32_t)(2 * step) ? (int32_t)((uint32_t)num / (2 * step)) : 1;
      return (int64_t)fit * Gs;
    };
    const int Ws = __builtin_amdgcn_readfirstlane(W);
    int next_fresh = 0;
    bool built = false;
    int k = 0;
    for (int s0 = 0; s0 < n_chunks; s0 += 64) {
      int4 rec = make_int4(0, 0, 0, 0);
      if (s0 + lane < n_chunks) rec = srec[s0 + lane];   // 64 chunk records per load, one per lane
      const int lim = min(64, n_chunks - s0);
      for (int i = 0; i < lim; ++i) {
        const int bh = __builtin_amdgcn_readlane(rec.x, i), ci = __builtin_amdgcn_readlane(rec.y, i);
        const int h = bh >> 16;
        int t0 = __builtin_amdgcn_readlane(rec.z, i);
        const int t1 = __builtin_amdgcn_readlane(rec.w, i);
        const uint32_t ds = (uint32_t)__builtin_amdgcn_readfirstlane((int)d_sum[h]);
        const uint32_t step = (uint32_t)Gs * ds;
        const int64_t fresh_fit = split ? fit_tokens(0, step) : INT64_MAX;   // what an untouched worker takes
        const int first_k = k;
        while (t0 < t1) {
          const bool fresh = next_fresh < Ws;
          if (fresh && P == 0) {
            // Untouched workers take the same number of tokens of this chunk each (the last one the rest),
            // and they are handed out in id order: up to 64 hand-outs at once, one per lane.
            const uint32_t R = (uint32_t)(t1 - t0);
            const uint32_t F = fresh_fit > (int64_t)R ? R : (uint32_t)fresh_fit;
            uint32_t cnt = (R + F - 1) / F;
            cnt = min(cnt, min((uint32_t)(Ws - next_fresh), 64u));
            cnt = (uint32_t)__builtin_amdgcn_readfirstlane((int)cnt);
            if ((uint32_t)lane < cnt) {
              const int lo = t0 + (int)((uint32_t)lane * F), hi = min(t1, lo + (int)F);
              const int w = next_fresh + lane, kk = k + lane;
              if (kk < n_max) {
                pieces[2 * (size_t)kk] = make_int4(ci, bh, lo, hi);
                pieces[2 * (size_t)kk + 1] = make_int4(w, 0, kk - first_k, 0);
              }
              wcount[w] = 1, loads[w] = (uint32_t)(hi - lo) * ds;
            }
            k += (int)cnt, next_fresh += (int)cnt;
            const uint64_t adv = (uint64_t)cnt * F;
            t0 = adv >= R ? t1 : t0 + (int)adv;
            continue;
          }
          uint32_t m, w;
          int64_t fit;
          if (fresh) {
            m = 0, w = (uint32_t)next_fresh++, fit = fresh_fit;
          } else {
            if (!built) {
              for (uint32_t sg = 0; sg < 64; ++sg) rescan(sg);
              built = true;
            }
            // least-loaded worker, lowest id among equals: segments are id ranges in lane order
            m = (uint32_t)__builtin_amdgcn_readfirstlane((int)wave_min_u32(segmin));
            const int sl = __builtin_ctzll(__ballot(segmin == m));
            w = (uint32_t)__builtin_amdgcn_readlane((int)segarg, sl);
            fit = split ? fit_tokens(m, step) : INT64_MAX;
          }
          int take = t1 - t0;
          if (fit < take) take = (int)fit;
          take = __builtin_amdgcn_readfirstlane(take);
          const int end = t0 + take;
          if (lane == 0) loads[w] = m + (uint32_t)take * ds;
          const uint32_t rank0 = fresh ? 0u : wcount[w];
          uint32_t np = 0;
          for (int lo = t0; lo < end;) {   // one piece per page it touches
            const int hi = P > 0 ? min(end, (lo / P + 1) * P) : end;
            if (k < n_max && lane == 0) {
              pieces[2 * (size_t)k] = make_int4(ci, bh, lo, hi);
              pieces[2 * (size_t)k + 1] = make_int4((int)w, (int)(rank0 + np), k - first_k, 0);
            }
            ++k, ++np, lo = hi;
          }
          if (lane == 0) wcount[w] = rank0 + np;
          if (!fresh) rescan(w >> seg_log2);
          t0 = end;
        }
        if (lane == 0) chunk_cnt[ci] = (uint32_t)(k - first_k);
      }
    }
    if (lane == 0) {
      if (k > n_max) atomicOr(&sh_status, kPlanOverflow), k = 0;
      sh_n_items = k;
    }
  }
  __syncthreads();
  const int n = sh_n_items;
  const bool overflow = (sh_status & kPlanOverflow) != 0;

  // ---- worker lists (CSR) and tile numbering ---------------------------------------------------------
  for (int w = tid; w < W; w += kPlanThreads) ex_wload[w] = overflow ? 0 : (int64_t)loads[w];
  if (overflow)
    for (int w = tid; w < 64 * seg; w += kPlanThreads) wcount[w] = 0;
  __syncthreads();
  block_exclusive_scan(wcount, W, red32);   // wcount[w] = first position of worker w, wcount[W] = n
  for (int ci = tid; ci < n_chunks; ci += kPlanThreads) chunk_base[ci] = overflow ? 0 : chunk_cnt[ci];
  __syncthreads();
  block_exclusive_scan(chunk_base, n_chunks, red32);   // tiles are numbered by (unit, first token) = chunk order

  // ---- launch slots -----------------------------------------------------------------------------------
  // As in the host planner: the tile kernel runs kWorkersPerGroup workers per workgroup, workgroup i runs on XCD
  // i % kXcds, and the even XCDs stream faster, so the heavier half of the workers takes their slots. Here the
  // half is found without a sort: the median load by bisection on its value (32 counts over the workgroup), then
  // every worker's rank among the heavier ones, among those at the median and among the rest (one scan over
  // per-thread counts). Inside a half workers keep id order (the host orders them by load: headers are not part
  // of the exported tables). loads[w] becomes the slot of worker w.
  const int per_w = (W + kPlanThreads - 1) / kPlanThreads;
  const bool slotted = c.g == 1 && !overflow && W % (2 * kXcds * kWorkersPerGroup) == 0 && per_w <= 4;
  if (slotted) {
    __shared__ uint32_t sh_cnt;
    const int w_lo = min(W, tid * per_w), w_hi = min(W, w_lo + per_w);
    uint32_t my[4] = {0, 0, 0, 0};
    for (int i = w_lo; i < w_hi; ++i) my[i - w_lo] = loads[i];
    auto count_above = [&](uint32_t thr, bool or_equal) -> uint32_t {   // workers with load > thr (>= thr)
      if (tid == 0) sh_cnt = 0;
      __syncthreads();
      uint32_t cnt = 0;
      for (int i = w_lo; i < w_hi; ++i) cnt += (my[i - w_lo] > thr || (or_equal && my[i - w_lo] == thr)) ? 1u : 0u;
      if (cnt) atomicAdd(&sh_cnt, cnt);
      __syncthreads();
      const uint32_t total = sh_cnt;
      __syncthreads();
      return total;
    };
    uint32_t lo = 0, hi = 0xffffffffu;   // the smallest T with at most W / 2 loads above it
    for (int it = 0; it < 32; ++it) {
      const uint32_t mid = lo + (hi - lo) / 2;
      if (count_above(mid, false) > (uint32_t)(W / 2)) lo = mid + 1;
      else hi = mid;
    }
    const uint32_t T = lo;
    const uint32_t n_above = count_above(T, false), n_extra = (uint32_t)(W / 2) - n_above;   // at T: the first n_extra join them
    uint32_t mine = 0;   // this thread's workers above T (low half), at T (high half)
    for (int i = w_lo; i < w_hi; ++i) mine += my[i - w_lo] > T ? 1u : (my[i - w_lo] == T ? 0x10000u : 0u);
    red32[tid] = mine;
    __syncthreads();
    for (int o = 1; o < kPlanThreads; o <<= 1) {   // inclusive scan of the packed counts (both stay below 2^16)
      const uint32_t add = tid >= o ? red32[tid - o] : 0;
      __syncthreads();
      red32[tid] += add;
      __syncthreads();
    }
    uint32_t run = tid > 0 ? red32[tid - 1] : 0;
    __syncthreads();   // red32 is free again
    for (int i = w_lo; i < w_hi; ++i) {
      const uint32_t above = run & 0xffffu, at = run >> 16, v = my[i - w_lo];
      int half, idx;   // position inside the heavier (0) or the lighter (1) half
      if (v > T) half = 0, idx = (int)above;
      else if (v == T && at < n_extra) half = 0, idx = (int)(n_above + at);
      else half = 1, idx = i - (int)(above + min(at, n_extra));
      const int grp = idx / kWorkersPerGroup;   // the half's workgroups in launch order
      const int wg = kXcds * (grp / (kXcds / 2)) + 2 * (grp % (kXcds / 2)) + half;
      loads[i] = (uint32_t)(wg * kWorkersPerGroup + idx % kWorkersPerGroup);
      run += v > T ? 1u : (v == T ? 0x10000u : 0u);
    }
    __syncthreads();
  }

  for (int k = tid; k < n; k += kPlanThreads) {
    const int4 pa = pieces[2 * (size_t)k], pb = pieces[2 * (size_t)k + 1];
    const int ci = pa.x, b = pa.y & 0xffff, h = pa.y >> 16, lo = pa.z, hi = pa.w;
    const int w = pb.x, rank = pb.y, in_chunk = pb.z;
    int32_t nb, size;
    chunk_shape(len[b], G, c.min_split, &nb, &size);
    const uint32_t u_first = cbase[b] + (uint32_t)(h * nb);
    const int u_beg = (int)chunk_base[u_first], u_end = (int)chunk_base[u_first + nb];
    const int n_u = u_end - u_beg;
    const int item = (int)chunk_base[ci] + in_chunk;
    const int pos = (int)wcount[w] + rank;
    int64_t row = b, in_row = lo;
    if (c.page_tokens > 0) {
      int32_t pg = block_table[(size_t)b * c.max_pages + lo / c.page_tokens];
      if (pg < 0 || pg >= c.n_pages) {
        atomicOr(&sh_status, kPlanBadPage);
        pg = 0;
      }
      row = pg, in_row = lo % c.page_tokens;
    }
    DecTile t;
    t.k_elem = row * c.row_tokens * c.RK + (int64_t)c.row_tokens * koff_r[h] + in_row * rk[h];
    t.v_elem = row * c.row_tokens * c.RV + (int64_t)c.row_tokens * voff_r[h] + in_row * rv[h];
    t.len = hi - lo;
    t.q_elem = c.g * (b * c.RK + koff_r[h]);
    t.o_elem = c.g * (b * c.RV + voff_r[h]);
    t.rk_rv = rk[h] | (rv[h] << 16);
    t.slot = n_u == 1 ? -1 : c.g * u_beg + (item - u_beg);
    t.g = c.g;
    t.slot_stride = n_u;
    t.b_end = b | (hi == len[b] ? (int32_t)0x80000000 : 0);
    wtiles[pos] = t;
    if (rank == 0) heads[slotted ? (int)loads[w] : w].first = t;
    ex_b[item] = b, ex_h[item] = h, ex_lo[item] = lo, ex_hi[item] = hi;
    ex_witems[pos] = item;
  }
  for (int w = tid; w < W; w += kPlanThreads) {
    const int begin = (int)wcount[w], count = (int)wcount[w + 1] - begin;
    DecWorker& hd = heads[slotted ? (int)loads[w] : w];
    hd.begin = begin, hd.count = count, hd.pad[0] = 0, hd.pad[1] = 0;
    if (count == 0) {
      DecTile z;
      memset(&z, 0, sizeof(z));
      hd.first = z;
    }
    ex_wptr[w] = begin;
  }
  if (tid == 0) ex_wptr[W] = n;
  int my_max = 0;
  for (int u = tid; u < n_units; u += kPlanThreads) {
    const int b = u / H, h = u % H;
    int32_t nb, size;
    chunk_shape(len[b], G, c.min_split, &nb, &size);
    const uint32_t u_first = cbase[b] + (uint32_t)(h * nb);
    const int u_beg = overflow ? 0 : (int)chunk_base[u_first], u_end = overflow ? 0 : (int)chunk_base[u_first + nb];
    const int n_u = u_end - u_beg;
    my_max = max(my_max, n_u);
    for (int j = 0; j < c.g; ++j) {
      const int first = c.g * u_beg + j * n_u;
      DecUnit r;
      r.tile_begin = first, r.tile_end = first + n_u;
      r.o_elem = c.g * (b * c.RV + voff_r[h]) + j * rv[h], r.rv = rv[h];
      units[(size_t)u * c.g + j] = r;
    }
    ex_uptr[u] = u_beg;
  }
  if (tid == 0) ex_uptr[n_units] = n;
  atomicMax(&sh_max_items, my_max);
  __syncthreads();
  if (tid == 0) {
    DevPlanHeader hd;
    hd.n_items = n, hd.max_items_per_unit = sh_max_items, hd.status = sh_status, hd.n_chunks = n_chunks;
    hd.total = (int64_t)total, hd.mean = sh_mean;
    *header = hd;
  }
}

}  // namespace fdc

using namespace fdc;

extern "C" {

static fdc_status plan_decode_device_body(const fdc_layout* lay, int layer, int batch, int max_pages,
                                          const fdc_plan_params* pr, fdc_plan** out) {
  const char* fn = "fdc_plan_decode_device";
  if (!out) FDC_FAIL(FDC_INVALID_ARG, "%s: out is NULL", fn);
  *out = nullptr;
  if (!lay || !pr) FDC_FAIL(FDC_INVALID_ARG, "%s: NULL argument", fn);
  if (layer < 0 || layer >= lay->L) FDC_FAIL(FDC_BAD_SHAPE, "%s: layer %d outside [0, %d)", fn, layer, lay->L);
  const bool paged = max_pages > 0;
  if (max_pages < 0) FDC_FAIL(FDC_BAD_SHAPE, "%s: max_pages must be 0 (dense cache) or positive", fn);
  if (batch <= 0 || batch > kPlanMaxBatch || (!paged && batch > lay->max_batch))
    FDC_FAIL(FDC_BAD_SHAPE, "%s: batch %d outside [1, %d]", fn, batch, paged ? kPlanMaxBatch : std::min(kPlanMaxBatch, lay->max_batch));
  if (pr->n_workers <= 0 || pr->n_workers > kPlanMaxWorkers)
    FDC_FAIL(FDC_INVALID_ARG, "%s: n_workers %d outside [1, %d]", fn, pr->n_workers, kPlanMaxWorkers);
  if (pr->softmax_cost <= 0) FDC_FAIL(FDC_INVALID_ARG, "%s: softmax_cost must be positive", fn);
  if (pr->granule <= 0 || pr->min_split <= 0)
    FDC_FAIL(FDC_INVALID_ARG, "%s: granule and min_split must be positive", fn);
  const int H = lay->H, W = pr->n_workers;
  if (H > kPlanMaxHeads) FDC_FAIL(FDC_BAD_SHAPE, "%s: more than %d heads; use fdc_plan_decode", fn, kPlanMaxHeads);
  const int64_t P = paged ? lay->max_seq : 0, G = pr->granule;
  if (paged && P % G != 0)
    FDC_FAIL(FDC_INVALID_ARG, "%s: the page size %d must be a multiple of the granule %d", fn, (int)P, pr->granule);
  const int64_t cap = paged ? P * max_pages : lay->max_seq;
  if (cap >= ((int64_t)1 << 30)) FDC_FAIL(FDC_BAD_SHAPE, "%s: sequences of up to %lld tokens; use fdc_plan_decode", fn, (long long)cap);
  const int32_t* rk = &lay->rk[(size_t)layer * H];
  const int32_t* rv = &lay->rv[(size_t)layer * H];
  int64_t D = 0, d_max = 0, d_min = INT64_MAX;
  for (int h = 0; h < H; ++h) {
    const int64_t d = (int64_t)rk[h] + rv[h] + pr->softmax_cost;
    D += d, d_max = std::max(d_max, d), d_min = std::min(d_min, d);
  }
  // what the kernel keeps in 32 bits: worker loads (at most the mean plus one step) and steps
  const int64_t mean_bound = ceil_div((int64_t)batch * cap * D, W) + G * d_max;
  if (mean_bound >= kPlanMaxLoad || 2 * G * d_max >= kPlanMaxLoad)
    FDC_FAIL(FDC_BAD_SHAPE, "%s: worker loads of up to %lld exceed the kernel's 32-bit range; use fdc_plan_decode", fn,
             (long long)mean_bound);
  const int64_t granules = ceil_div(cap, G);
  const int64_t chunks_max = (int64_t)batch * H * std::min<int64_t>(pr->min_split, granules);
  if (chunks_max > kPlanMaxChunks)
    FDC_FAIL(FDC_BAD_SHAPE, "%s: up to %lld chunks, the kernel sorts at most %d; use fdc_plan_decode", fn,
             (long long)chunks_max, kPlanMaxChunks);
  // Pieces. A unit is never cut finer than the granule (pages are multiples of it). And: every hand-out
  // that leaves part of its chunk behind fills its worker to within half a step of the mean; once the
  // least-loaded worker is that full all are, at most W * G * d_max / 2 of work is left and every further
  // hand-out takes at least G * d_min of it.
  const int64_t by_granule = (int64_t)batch * H * granules;
  const int64_t by_fill = chunks_max + W + ceil_div((int64_t)W * d_max, 2 * d_min) +
                          (paged ? (int64_t)batch * H * (max_pages - 1) : 0);
  const int64_t n_max = std::max<int64_t>(1, std::min(by_granule, by_fill));

  std::unique_ptr<fdc_plan> holder(new fdc_plan());
  fdc_plan* p = holder.get();
  p->kind = 0, p->on_device = true, p->layer = layer, p->batch = batch, p->H = H, p->n_workers = W;
  p->n_units = batch * H, p->G = lay->G, p->lay = lay, p->RK = lay->RK(layer), p->RV = lay->RV(layer);
  p->total_q_rows = batch, p->n_merge_units = p->n_units * p->G, p->n_max = n_max;
  p->max_unit_granules = granules;   // cuts fall on granule multiples (pages are multiples of the granule)
  p->d_sum.resize(H);
  for (int h = 0; h < H; ++h) p->d_sum[h] = (int64_t)rk[h] + rv[h] + pr->softmax_cost;

  DevPlanConst c;
  std::memset(&c, 0, sizeof(c));
  c.batch = batch, c.H = H, c.W = W, c.granule = pr->granule, c.min_split = pr->min_split, c.split = pr->split ? 1 : 0;
  c.softmax_cost = pr->softmax_cost, c.g = lay->G, c.row_tokens = lay->max_seq, c.page_tokens = (int32_t)P;
  c.max_pages = max_pages, c.n_pages = lay->max_batch, c.seq_cap = (int32_t)cap, c.n_max = (int32_t)n_max;
  c.RK = p->RK, c.RV = p->RV, c.n_merge_units = p->n_merge_units;
  c.n_pad = 2;
  while (c.n_pad < chunks_max) c.n_pad *= 2;
  c.seg_log2 = 0;
  while ((64 << c.seg_log2) < W) ++c.seg_log2;
  const size_t W_pad = (size_t)64 << c.seg_log2;
  // LDS
  size_t lo = 0;
  auto lds = [&](size_t bytes) { const size_t at = lo; lo += (bytes + 15) / 16 * 16; return (uint32_t)at; };
  c.lds_keys = lds(std::max<size_t>((size_t)c.n_pad * 8, ((size_t)chunks_max + 1) * 4));
  c.lds_loads = lds(W_pad * 4);
  c.lds_wcount = lds((W_pad + 1) * 4);
  c.lds_len = lds((size_t)batch * 4);
  c.lds_cbase = lds(((size_t)batch + 1) * 4);
  c.lds_dsum = lds((size_t)H * 4);
  c.lds_red = lds((size_t)kPlanThreads * 8);
  c.lds_bytes = (uint32_t)lo;
  if (lo + 64 > kPlanMaxLds) {
    delete p;
    FDC_FAIL(FDC_BAD_SHAPE, "%s: the problem needs %zu bytes of LDS (limit %zu); use fdc_plan_decode", fn, lo, kPlanMaxLds);
  }
  // workspace
  size_t wo = 0;
  auto region = [&](size_t bytes) { const size_t at = (wo + 255) / 256 * 256; wo = at + std::max<size_t>(bytes, 16); return at; };
  const size_t const_bytes = sizeof(DevPlanConst) + (size_t)4 * H * sizeof(int32_t);
  region(const_bytes);
  c.off_header = region(sizeof(DevPlanHeader));
  c.off_items = region((size_t)n_max * sizeof(DecTile));
  c.off_units = region((size_t)p->n_merge_units * sizeof(DecUnit));
  c.off_workers = region((size_t)W * sizeof(DecWorker));
  c.off_lens = region((size_t)batch * sizeof(int32_t));
  c.off_export = region(export_offsets(n_max, p->n_units, W).bytes);
  c.off_srec = region((size_t)c.n_pad * sizeof(int4));
  c.off_chunk_cnt = region((size_t)c.n_pad * sizeof(uint32_t));
  c.off_pieces = region((size_t)n_max * 2 * sizeof(int4));
  p->off_header = c.off_header, p->off_export = c.off_export, p->lds_bytes = c.lds_bytes;
  p->off_items = c.off_items, p->off_units = c.off_units, p->off_worker_ptr = p->off_worker_items = c.off_workers;
  p->off_lens = c.off_lens;
  p->off_partials = (wo + 255) / 256 * 256;
  p->partial_bytes = (size_t)n_max * p->G * kPartialStride * sizeof(float);
  p->workspace_bytes = p->off_partials + p->partial_bytes;
  // the constants are the plan's image: fdc_plan_upload puts them at the start of the workspace
  p->image.resize(const_bytes);
  std::memcpy(p->image.data(), &c, sizeof(c));
  int32_t* tab = reinterpret_cast<int32_t*>(p->image.data() + sizeof(c));
  const int32_t* koff_r = &lay->koff_r[(size_t)layer * (H + 1)];
  const int32_t* voff_r = &lay->voff_r[(size_t)layer * (H + 1)];
  for (int h = 0; h < H; ++h) tab[h] = rk[h], tab[H + h] = rv[h], tab[2 * H + h] = koff_r[h], tab[3 * H + h] = voff_r[h];
  *out = holder.release();
  return FDC_OK;
}

fdc_status fdc_plan_decode_device(const fdc_layout* lay, int layer, int batch, int max_pages,
                                  const fdc_plan_params* pr, fdc_plan** out) {
  return guarded("fdc_plan_decode_device", [&] { return plan_decode_device_body(lay, layer, batch, max_pages, pr, out); });
}

fdc_status fdc_plan_decode_run(fdc_plan* const* plans, void* const* workspaces, int n_plans, const int32_t* seq_len,
                               const int32_t* block_table, void* stream) {
  const char* fn = "fdc_plan_decode_run";
  if (!plans || !workspaces || !seq_len) FDC_FAIL(FDC_INVALID_ARG, "%s: NULL argument", fn);
  if (n_plans <= 0 || n_plans > kPlanMaxLayersPerLaunch)
    FDC_FAIL(FDC_BAD_SHAPE, "%s: %d plans, a launch takes 1 to %d", fn, n_plans, kPlanMaxLayersPerLaunch);
  DevPlanLaunch launch;
  std::memset(&launch, 0, sizeof(launch));
  size_t lds_bytes = 0;
  for (int i = 0; i < n_plans; ++i) {
    const fdc_plan* p = plans[i];
    if (!p || !workspaces[i]) FDC_FAIL(FDC_INVALID_ARG, "%s: plan or workspace %d is NULL", fn, i);
    if (p->kind != 0 || !p->on_device) FDC_FAIL(FDC_INVALID_ARG, "%s: plan %d was not made by fdc_plan_decode_device", fn, i);
    if (p->batch != plans[0]->batch) FDC_FAIL(FDC_BAD_SHAPE, "%s: plan %d is for batch %d, plan 0 for %d", fn, i, p->batch, plans[0]->batch);
    const DevPlanConst* c = reinterpret_cast<const DevPlanConst*>(p->image.data());
    const DevPlanConst* c0 = reinterpret_cast<const DevPlanConst*>(plans[0]->image.data());
    if (c->page_tokens != c0->page_tokens || c->max_pages != c0->max_pages)
      FDC_FAIL(FDC_BAD_SHAPE, "%s: plan %d and plan 0 differ in page size or pages per sequence", fn, i);
    if (c->page_tokens > 0 && !block_table) FDC_FAIL(FDC_INVALID_ARG, "%s: paged plans need block_table", fn);
    if ((reinterpret_cast<uintptr_t>(workspaces[i]) & 255u) != 0)
      FDC_FAIL(FDC_BAD_ALIGNMENT, "%s: workspace %d must be 256-byte aligned", fn, i);
    for (int j = 0; j < i; ++j)
      if (workspaces[j] == workspaces[i]) FDC_FAIL(FDC_INVALID_ARG, "%s: plans %d and %d share a workspace", fn, j, i);
    launch.ws[i] = static_cast<unsigned char*>(workspaces[i]);
    lds_bytes = std::max<size_t>(lds_bytes, p->lds_bytes);
  }
  if (lds_bytes > 64 * 1024) {
    static std::mutex mu;
    static std::vector<int> done;
    int dev = 0;
    FDC_HIP_CHECK(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(mu);
    if (std::find(done.begin(), done.end(), dev) == done.end()) {
      FDC_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(plan_decode_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)kPlanMaxLds - 64));
      try {
        done.push_back(dev);
      } catch (...) {   // not remembered: the attribute is simply set again next time
      }
    }
  }
  hipLaunchKernelGGL(plan_decode_kernel, dim3(n_plans), dim3(kPlanThreads), lds_bytes, static_cast<hipStream_t>(stream),
                     launch, seq_len, block_table);
  FDC_HIP_CHECK(hipGetLastError());
  for (int i = 0; i < n_plans; ++i) plans[i]->downloaded = false;
  return FDC_OK;
}

static fdc_status plan_download_body(fdc_plan* p, const void* workspace, void* stream) {
  const char* fn = "fdc_plan_download";
  if (!p || !workspace) FDC_FAIL(FDC_INVALID_ARG, "%s: NULL argument", fn);
  if (p->kind != 0 || !p->on_device) FDC_FAIL(FDC_INVALID_ARG, "%s: not a plan made by fdc_plan_decode_device", fn);
  const unsigned char* ws = static_cast<const unsigned char*>(workspace);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t n_max = p->n_max;
  const int W = p->n_workers;
  const ExportOffsets eo = export_offsets(n_max, p->n_units, W);
  DevPlanHeader hd;
  std::vector<unsigned char> ex(eo.bytes);
  FDC_HIP_CHECK(hipMemcpyAsync(&hd, ws + p->off_header, sizeof(hd), hipMemcpyDeviceToHost, st));
  FDC_HIP_CHECK(hipMemcpyAsync(ex.data(), ws + p->off_export, eo.bytes, hipMemcpyDeviceToHost, st));
  FDC_HIP_CHECK(hipStreamSynchronize(st));
  if (hd.n_items < 0 || hd.n_items > n_max) FDC_FAIL(FDC_INVALID_ARG, "%s: the workspace holds no plan of this shape (run fdc_plan_decode_run first)", fn);
  const size_t n = (size_t)hd.n_items;
  auto i32 = [&](size_t off) { return reinterpret_cast<const int32_t*>(ex.data() + off); };
  p->item_b.assign(i32(eo.item_b), i32(eo.item_b) + n);
  p->item_h.assign(i32(eo.item_h), i32(eo.item_h) + n);
  p->item_lo.assign(i32(eo.item_lo), i32(eo.item_lo) + n);
  p->item_hi.assign(i32(eo.item_hi), i32(eo.item_hi) + n);
  p->worker_items.assign(i32(eo.worker_items), i32(eo.worker_items) + n);
  p->unit_item_ptr.assign(i32(eo.unit_item_ptr), i32(eo.unit_item_ptr) + p->n_units + 1);
  p->worker_ptr.assign(i32(eo.worker_ptr), i32(eo.worker_ptr) + W + 1);
  const int64_t* wl = reinterpret_cast<const int64_t*>(ex.data() + eo.worker_load);
  p->worker_load.assign(wl, wl + W);
  p->item_cost.resize(n);
  for (size_t i = 0; i < n; ++i) {
    if (p->item_h[i] < 0 || p->item_h[i] >= p->H) FDC_FAIL(FDC_INVALID_ARG, "%s: the workspace holds no plan of this shape", fn);
    p->item_cost[i] = (int64_t)(p->item_hi[i] - p->item_lo[i]) * p->d_sum[p->item_h[i]];
  }
  p->max_items_per_unit = hd.max_items_per_unit;
  p->downloaded = true;
  if (hd.status & kPlanOverflow) FDC_FAIL(FDC_BAD_SHAPE, "%s: the planner ran out of piece slots; nothing was scheduled", fn);
  if (hd.status & kPlanBadLength)
    FDC_FAIL(FDC_BAD_SHAPE, "%s: a sequence length on the device was outside [0, cap]; it was planned clamped", fn);
  if (hd.status & kPlanBadPage)
    FDC_FAIL(FDC_BAD_SHAPE, "%s: a block-table entry on the device was outside the layout's pages; page 0 was used", fn);
  return FDC_OK;
}

fdc_status fdc_plan_download(fdc_plan* p, const void* workspace, void* stream) {
  return guarded("fdc_plan_download", [&] { return plan_download_body(p, workspace, stream); });
}

}  // extern "C"
