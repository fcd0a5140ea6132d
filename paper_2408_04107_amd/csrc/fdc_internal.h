// Internal declarations shared by the host side and the kernels of libfdc.
#pragma once

#include <atomic>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <exception>
#include <memory>
#include <new>
#include <string>
#include <vector>

#include "fdc.h"

namespace fdc {

// ---- error text ---------------------------------------------------------------------------
void set_error(const char* fmt, ...);
#define FDC_FAIL(code, ...)        \
  do {                             \
    ::fdc::set_error(__VA_ARGS__); \
    return (code);                 \
  } while (0)

#define FDC_HIP_CHECK(expr)                                                        \
  do {                                                                             \
    hipError_t e_ = (expr);                                                        \
    if (e_ != hipSuccess) FDC_FAIL(FDC_HIP_ERROR, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

// Runs the body of an entry point that allocates host memory (std::vector, std::string): no C++
// exception may cross the C boundary, so a failed allocation becomes an error status with text.
template <typename F>
inline fdc_status guarded(const char* fn, F&& body) noexcept {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    set_error("%s: out of host memory", fn);
  } catch (const std::exception& e) {
    set_error("%s: %s", fn, e.what());
  } catch (...) {
    set_error("%s: unknown failure", fn);
  }
  return FDC_INVALID_ARG;
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int64_t round_up(int64_t a, int64_t m) { return ceil_div(a, m) * m; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- device-side descriptors (plain structs copied into the workspace) ----------------------

// One decode tile: a token range of one (sequence, head) unit. 48 bytes.
struct DecTile {
  int64_t k_elem;   // element offset of the tile's first K' row inside the layer's K' buffer
  int64_t v_elem;   // same for V'
  int32_t len;      // tokens in the tile (> 0)
  int32_t q_elem;   // element offset of q'_h in q_lat  (b * RK + koff_r[h])
  int32_t o_elem;   // element offset of o'_h in o_lat  (b * RV + voff_r[h])
  int32_t rk_rv;    // rk | rv << 16
  int32_t slot;     // partial-state slot, or -1: the unit has one tile, write the normalised output
  int32_t g;        // query heads that share the unit's K'/V' (1 = multi-head); query j of the group
                    // reads q' at q_elem + j * rk, writes o' at o_elem + j * rv and uses partial slot
                    // slot + j * slot_stride
  int32_t slot_stride;  // tiles of the unit
  int32_t b_end;        // the sequence (bits 0..30); bit 31 set when the tile ends at the sequence's planned
                        // length, i.e. it is the tile that shrinks when the call is given shorter actual lengths
};

// Length of a tile when the call passes the actual sequence lengths (device int32 [batch], each in the
// last granule of the planned length): tiles that end the sequence give up planned - actual tokens.
// Never longer than planned and never empty, whatever the array holds.
#ifdef __HIPCC__
__device__ inline int32_t dec_tile_len(const DecTile& t, const int32_t* planned_len, const int32_t* seq_len) {
  if (seq_len == nullptr || t.b_end >= 0) return t.len;
  const int32_t b = t.b_end & 0x7fffffff;
  const int32_t cut = planned_len[b] - seq_len[b];
  return cut <= 0 ? t.len : (t.len - cut < 1 ? 1 : t.len - cut);
}
#endif
static_assert(sizeof(DecTile) == 48, "DecTile layout");

// Launch geometry the host planner relies on when it orders the worker headers by launch slot.
constexpr int kXcds = 8;              // accelerator dies (XCDs) of the GPU; workgroups are dealt to them in turn
constexpr int kWorkersPerGroup = 4;   // wavefronts (workers) per workgroup of both decode tile kernels

// What a decode worker (one wavefront) reads first: how many tiles it has, where the rest of them
// are in the worker-ordered tile array, and its first tile inline, so that the cache stream starts
// after a single dependent load. 64 bytes.
struct DecWorker {
  int32_t begin;   // index of the worker's first tile in the worker-ordered tile array
  int32_t count;   // tiles of this worker
  int32_t pad[2];
  DecTile first;
};
static_assert(sizeof(DecWorker) == 64, "DecWorker layout");

// One (sequence, head) unit for the split-K merge. 16 bytes.
struct DecUnit {
  int32_t tile_begin, tile_end;  // partial slots of the unit
  int32_t o_elem;
  int32_t rv;
};

// Cache element of an E2M1 layout: a byte holds two codes, so buffers are addressed in bytes = elements / 2.
struct fp4_t {
  uint8_t pair;
};

// Tokens of a K'/V' block the prefill kernel stages at a time; a page holds a whole number of them.
constexpr int kPrefillBlockTokens = 128;

// Partial state of a tile: m, l, 2 pad floats, acc[rv <= 128].
constexpr int kPartialStride = 132;

// One prefill task: query rows [q0, q1) of one (sequence, head) unit. 64 bytes.
struct PreTask {
  int64_t k_elem;    // element offset of the unit's first K' row
  int64_t v_elem;
  int64_t q_elem;    // element offset of (row q0, head column 0) in q_lat [T, RK]
  int64_t o_elem;    // element offset of (row q0, head column 0) in o_lat [T, RV]
  int32_t rows;      // q1 - q0
  int32_t pos0;      // absolute position of row q0 in the sequence (kv_len - q_len + q0)
  int32_t kv_len;    // keys of the sequence
  int32_t rk_rv;     // rk | rv << 16
  int32_t ldq;       // RK (row stride of q_lat)
  int32_t ldo;       // RV
  int32_t page_tokens;  // 0: k_elem / v_elem address the unit's rows [0, kv_len) directly. P > 0: the cache
                        // is paged; tokens i*P .. of the sequence sit in page page_table[page_first + i], and
                        // k_elem / v_elem are the head's offsets inside a page
  int32_t page_first;   // index of the sequence's first entry in the plan's page table
};
static_assert(sizeof(PreTask) == 64, "PreTask layout");

// Resident workgroups per compute unit of the prefill kernel (occupancy query).
fdc_status prefill_blocks_per_cu(int* nb);

// Grouped-query decode tile kernel (fdc_decode_gqa.hip): resident workers per compute unit, and the
// launch. Same tables, partial slots and outputs as the multi-head tile kernel.
struct DecWorker;
fdc_status decode_gqa_workers_per_cu(int* waves);

}  // namespace fdc

#ifdef __HIPCC__
#include <hip/hip_runtime.h>
namespace fdc {
fdc_status launch_decode_gqa(const DecWorker* heads, const DecTile* wtiles, const float* q_lat, const void* kc,
                             const void* vc, bool e4m3, float scale, float* o_lat, float* partials, int n_workers,
                             const int32_t* planned_len, const int32_t* seq_len, hipEvent_t ev0, hipEvent_t ev1,
                             hipStream_t st);
}
#endif

// ---- host objects ---------------------------------------------------------------------------
struct fdc_layout {
  int L, H, d_model, d_head, max_batch, max_seq;
  int G = 1;  // query heads per key/value head
  fdc_dtype dtype;
  int elem_bits;   // bits per cached element
  std::vector<int32_t> rk, rv;          // [L*H]
  std::vector<int32_t> koff_r, voff_r;  // [L*(H+1)]
  std::vector<int64_t> koff, voff;      // [L*H]
  std::vector<int64_t> k_elems, v_elems;  // [L]
  int RK(int l) const { return koff_r[(size_t)l * (H + 1) + H]; }
  int RV(int l) const { return voff_r[(size_t)l * (H + 1) + H]; }
};

namespace fdc {
// Process-wide serial numbers of plans (never 0, never reused): what tells a cached copy of a plan's
// tables from the tables of another plan that happens to live at the same address.
inline uint64_t next_plan_serial() {
  static std::atomic<uint64_t> counter{0};
  return ++counter;
}
}  // namespace fdc

struct fdc_plan {
  const uint64_t serial = fdc::next_plan_serial();
  int kind;  // 0 decode, 1 prefill
  int layer, batch, H, n_workers, n_units;
  int G = 1;            // query heads per key/value head of the layout the plan was made for
  int n_merge_units = 0;  // decode: records of the split-K merge (units x query heads of a group)
  const fdc_layout* lay;  // identity check only (the plan copies what it needs)
  int RK, RV;
  int64_t total_q_rows;   // prefill: T
  int max_items_per_unit = 0;  // decode: most tiles any unit was cut into
  int min_items_per_unit = 0;  // decode: fewest (empty units count as 0)
  // exported tables
  std::vector<int32_t> item_b, item_h, item_lo, item_hi, unit_item_ptr, worker_ptr, worker_items, br;
  std::vector<int64_t> item_cost, worker_load;
  // device image: packed tables, copied verbatim by fdc_plan_upload
  std::vector<unsigned char> image;
  size_t off_items, off_units, off_worker_ptr, off_worker_items;  // byte offsets inside image
  size_t off_lens = 0;         // decode: int32 planned sequence lengths [batch], inside image
  size_t off_pages = 0;        // prefill over a paged cache: int32 page table [batch * max_pages], inside image
  size_t off_partials, partial_bytes;                             // decode only, after the image
  size_t workspace_bytes;
  // Decode plans made on the device (fdc_plan_decode_device): the tables above stay empty until
  // fdc_plan_download; `image` holds only the constants of the planner kernel, and the regions of the
  // workspace are sized for n_max pieces, an upper bound known without the sequence lengths.
  bool on_device = false, downloaded = false;
  int64_t n_max = 0;
  int64_t max_unit_granules = 0;   // most pieces one unit can be cut into: ceil(capacity / granule)
  std::vector<int64_t> d_sum;   // per head, for item_cost after a download
  size_t off_header = 0, off_export = 0, lds_bytes = 0;
};
