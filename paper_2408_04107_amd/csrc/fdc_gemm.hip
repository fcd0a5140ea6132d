// The three projection-type calls of the hot path (Section 2 of the paper):
//   fdc_project_latent_kv   K' = x A_k, V' = x A_v, written into the ragged cache
//   fdc_absorb_query        q'_h = q_h B_k^T                      (grouped over heads)
//   fdc_absorb_output       M = B_v W_o (grouped, once) and y = o' M
// All four products have the form C[m, n] = sum_k A[m, k] * B[n, k] with both operands contiguous
// along k, so one bf16 MFMA kernel (fp32 accumulation) serves them and only the addressing of a
// group and the epilogue differ. FDC_F32 layouts use a plain fp32 kernel (validation shapes).
#include <hip/hip_runtime.h>

#include <climits>

#include <algorithm>
#include <mutex>
#include <utility>
#include <vector>

#include "fdc_internal.h"

namespace fdc {

constexpr int kMaxHeads = 128;

// A launch with more than 64 KiB of dynamic LDS needs the kernel's limit raised first, once per
// kernel and device. Kernels of one signature share a function-pointer type, so the record is
// keyed by the pointer's value, not by a per-template static.
static hipError_t ensure_dynamic_lds(const void* kern, size_t bytes) {
  static std::mutex mu;
  static std::vector<std::pair<const void*, int>> done;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> lock(mu);
  for (const auto& d : done)
    if (d.first == kern && d.second == dev) return hipSuccess;
  e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess) done.emplace_back(kern, dev);
  return e;
}

// Compute units of the current device (cached per device).
static hipError_t device_compute_units(int* cus) {
  static std::mutex mu;
  static std::vector<std::pair<int, int>> known;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> lock(mu);
  for (const auto& d : known)
    if (d.first == dev) {
      *cus = d.second;
      return hipSuccess;
    }
  e = hipDeviceGetAttribute(cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e == hipSuccess) known.emplace_back(dev, *cus);
  return e;
}

enum GemmMode { kPlain = 0, kProject = 1, kAbsorbQuery = 2, kFold = 3 };

struct GemmArgs {
  const void* A;
  const void* B;
  void* C;
  void* C2;  // project: the V' cache
  int64_t lda, ldb, ldc;
  int M, N, K;
  int nt;    // column tiles of the large kernel (of the widest group)
  int split_from;  // large kernel: blocks from this one on each take half (128 rows) of a tile
  int mode;
  int H, d_head, max_seq, max_batch;
  int32_t* fault;  // cache writers: device word that collects kFaultBatch / kFaultPos (may be NULL)
  int G;     // query heads per key/value head: grouped products run over the H * G query heads
  int RK, RV;
  const int32_t* tok_batch;
  const int32_t* tok_pos;
  int v_only;             // project: B holds only the V' rows, every column goes to the V' cache
  int cache_fp8;          // project: the caches hold E4M3 codes (one byte per element) instead of bf16
  int cache_fp4;          // project: the caches hold E2M1 codes, two per byte (even column in the low nibble)
  const float* rope_cos;  // post-RoPE path: [n_pos, d_head / 2]
  const float* rope_sin;
  int n_pos;
  int32_t koff_r[kMaxHeads + 1];
  int32_t voff_r[kMaxHeads + 1];
};

// Per-group view: which rows/columns this z-slice multiplies.
struct Group {
  int64_t a_off, b_off, c_off;
  int N;
};

__device__ __forceinline__ Group group_of(const GemmArgs& g, int z) {
  Group r{0, 0, 0, g.N};
  // z is a QUERY head; it uses the factors of key/value head h = z / G and is the j-th of its group
  const int h = z / g.G, j = z % g.G;
  if (g.mode == kAbsorbQuery) {  // A = q[:, z, :], B = Bk rows of head h, C = q_lat columns of query head z
    r.N = g.koff_r[h + 1] - g.koff_r[h];
    r.a_off = (int64_t)z * g.d_head;
    r.b_off = (int64_t)g.koff_r[h] * g.d_head;
    r.c_off = g.G * g.koff_r[h] + j * r.N;
  } else if (g.mode == kFold) {  // A = Wo_t[:, z*d_h ..], B = Bv rows of head h, C = Mt columns of query head z
    r.N = g.voff_r[h + 1] - g.voff_r[h];
    r.a_off = (int64_t)z * g.d_head;
    r.b_off = (int64_t)g.voff_r[h] * g.d_head;
    r.c_off = g.G * g.voff_r[h] + j * r.N;
  }
  return r;
}

__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);  // round to nearest, ties to even
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

template <typename T>
__device__ __forceinline__ void store_out(T* p, float v);
template <>
__device__ __forceinline__ void store_out<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_out<uint16_t>(uint16_t* p, float v) { *p = f32_to_bf16(v); }

// One cache element: bf16, or the E4M3 code of the value saturated to +-448 (v_cvt_pk_fp8_f32 rounds
// to nearest even and would turn larger values into NaN).
// Two values -> one byte of E2M1 codes (v_cvt_scalef32_pk_fp4_f32 with scale 1: round to nearest even;
// the inputs are clamped to the format's range first): lo in bits 3..0, hi in bits 7..4.
__device__ __forceinline__ uint32_t fp4_pair(float lo, float hi) {
  const float a = fminf(fmaxf(lo, -6.f), 6.f), b = fminf(fmaxf(hi, -6.f), 6.f);
  return __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, a, b, 1.0f, 0) & 0xffu;
}

// E2M1 caches: every caller has neighbouring lanes hold neighbouring columns of one row (the even
// column in the even lane), and a row's two lanes take the same branches, so the even lane fetches its
// neighbour's value and writes the byte they share.
__device__ __forceinline__ void store_cache(const GemmArgs& g, void* cache, int64_t e, float v) {
  if (g.cache_fp4) {
    const float right = __shfl_xor(v, 1);
    if ((threadIdx.x & 1) == 0) static_cast<uint8_t*>(cache)[e >> 1] = (uint8_t)fp4_pair(v, right);
  } else if (g.cache_fp8) {
    const float c = fminf(fmaxf(v, -448.f), 448.f);
    static_cast<uint8_t*>(cache)[e] = (uint8_t)(__builtin_amdgcn_cvt_pk_fp8_f32(c, 0.f, 0u, false) & 0xffu);
  } else {
    static_cast<uint16_t*>(cache)[e] = f32_to_bf16(v);
  }
}

// Destination token of input row m of a cache writer. Rows whose tok_batch / tok_pos lie outside
// the cache are skipped by every writer (nothing is stored for them) and noted in the caller's
// status word; the indices are device data, so no host check can catch them.
constexpr int kFaultBatch = 1, kFaultPos = 2;
__device__ __forceinline__ bool token_dst(const GemmArgs& g, int m, int* b, int* pos) {
  *b = g.tok_batch[m], *pos = g.tok_pos[m];
  const bool b_ok = (unsigned)*b < (unsigned)g.max_batch, p_ok = (unsigned)*pos < (unsigned)g.max_seq;
  if (b_ok && p_ok) return true;
  if (g.fault) atomicOr(g.fault, (b_ok ? 0 : kFaultBatch) | (p_ok ? 0 : kFaultPos));
  return false;
}

// Cache element for output column n of the concatenated [K heads | V heads] projection.
// Returns the buffer (0 = K', 1 = V') and the element offset for token (b, pos).
__device__ __forceinline__ int64_t project_dst(const GemmArgs& g, int n, int b, int pos, int* side) {
  const int s = g.v_only ? 1 : n >= g.RK;
  const int c = (s && !g.v_only) ? n - g.RK : n;
  const int32_t* off_r = s ? g.voff_r : g.koff_r;
  int lo = 0, hi = g.H;  // largest h with off_r[h] <= c
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (off_r[mid] <= c) lo = mid; else hi = mid;
  }
  const int r = off_r[lo + 1] - off_r[lo];
  const int R = s ? g.RV : g.RK;
  *side = s;
  return (int64_t)b * g.max_seq * R + (int64_t)g.max_seq * off_r[lo] + (int64_t)pos * r + (c - off_r[lo]);
}

// ---- fp32 reference-quality kernel for FDC_F32 layouts -----------------------------------------
template <typename TC>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const GemmArgs g) {
  const Group gr = group_of(g, blockIdx.z);
  const int n = blockIdx.x * 16 + threadIdx.x % 16;
  const int m = blockIdx.y * 16 + threadIdx.x / 16;
  if (m >= g.M || n >= gr.N) return;
  const float* a = static_cast<const float*>(g.A) + gr.a_off + (int64_t)m * g.lda;
  const float* b = static_cast<const float*>(g.B) + gr.b_off + (int64_t)n * g.ldb;
  float acc = 0.f;
  for (int k = 0; k < g.K; ++k) acc = fmaf(a[k], b[k], acc);
  if (g.mode == kProject) {
    int side, b, pos;
    if (!token_dst(g, m, &b, &pos)) return;
    const int64_t e = project_dst(g, n, b, pos, &side);
    static_cast<float*>(side ? g.C2 : g.C)[e] = acc;
  } else {
    store_out(static_cast<TC*>(g.C) + gr.c_off + (int64_t)m * g.ldc + n, acc);
  }
}

// ---- bf16 MFMA kernel --------------------------------------------------------------------------
// Workgroup tile 256 x 128, k step 64, four waves in a 2 x 2 grid, each wave 128 x 64 as 4 x 2
// v_mfma_f32_32x32x16_bf16 tiles (128 accumulator registers). Both operands are staged through LDS
// with rows padded by 16 bytes; fragments are read with one 16-byte LDS load per lane (8
// consecutive k of one row). The next k step is fetched into registers while the current one is
// multiplied, so a stage has 64 MFMAs per wave between its two barriers and two workgroups per
// compute unit cover each other's global-load latency.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2g __attribute__((ext_vector_type(2)));
typedef float f32x2g __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 256, BN = 128, BK = 64;
constexpr int kLdsRow = BK + 8;  // elements per padded LDS row (144 bytes)

__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {  // v_cvt_pk_bf16_f32 (round to nearest even)
  union { bf16x2g v; uint32_t u; } r;
  r.v = __builtin_convertvector(f32x2g{lo, hi}, bf16x2g);
  return r.u;
}

template <typename TA>
__device__ __forceinline__ u32x4 load_chunk(const TA* p);  // 8 consecutive elements -> 8 bf16
template <>
__device__ __forceinline__ u32x4 load_chunk<uint16_t>(const uint16_t* p) {
  return *reinterpret_cast<const u32x4*>(p);
}
template <>
__device__ __forceinline__ u32x4 load_chunk<float>(const float* p) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  return u32x4{cvt_pk_bf16(a.x, a.y), cvt_pk_bf16(a.z, a.w), cvt_pk_bf16(b.x, b.y), cvt_pk_bf16(b.z, b.w)};
}

template <typename TA, typename TC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void gemm_bf16_kernel(const GemmArgs g) {
  const Group gr = group_of(g, blockIdx.z);
  // Tile order. Workgroups are dealt round-robin to the 8 XCDs (each with its own L2), so the
  // linear id is first turned into "XCD-major" order: XCD x walks the contiguous tile range
  // [x * T/8, (x+1) * T/8). Inside that range tiles go down 8 row-tiles before moving to the next
  // column tile, so the ~64 workgroups resident on one XCD form an 8 x 8 patch that shares its A
  // and B panels through that XCD's L2 while all of them advance along k together.
  const int mt = (g.M + BM - 1) / BM, nt = g.nt;
  const int tiles = mt * nt, per_xcd = (tiles + 7) / 8;
  const int lin = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (lin >= tiles) return;
  constexpr int GM = 8;
  const int band = lin / (GM * nt), in_band = lin % (GM * nt);
  const int band_rows = min(GM, mt - band * GM);
  const int tm = band * GM + in_band % band_rows, tn = in_band / band_rows;
  const int m0 = tm * BM, n0 = tn * BN;
  if (n0 >= gr.N) return;
  __shared__ __attribute__((aligned(16))) uint16_t lds_a[BM * kLdsRow];
  __shared__ __attribute__((aligned(16))) uint16_t lds_b[BN * kLdsRow];

  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int wm = (wave / 2) * 128, wn = (wave % 2) * 64;
  const TA* A = static_cast<const TA*>(g.A) + gr.a_off;
  const uint16_t* B = static_cast<const uint16_t*>(g.B) + gr.b_off;

  // staging: a row of the stage is 8 chunks of 8 elements; 8 lanes per row, 32 rows per sweep.
  // The block's row panels are raw buffers that end with the last valid row, so rows past M / N
  // read zeros through the hardware range check and a stage needs no address arithmetic: the lane's
  // byte offsets are fixed and k0 goes into the scalar offset. Only the last, partial k stage
  // (K not a multiple of 64) compares k.
  constexpr int SA = BM / 32, SB = BN / 32;
  constexpr int ES = (int)sizeof(TA);
  const int s_row = tid / 8, s_kc = (tid % 8) * 8;
  const int a_rows = min(BM, g.M - m0), b_rows = min(BN, gr.N - n0);
  const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<TA*>(A + (int64_t)m0 * g.lda), 0, (int)(((int64_t)(a_rows - 1) * g.lda + g.K) * ES), 0x00020000);
  const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(B + (int64_t)n0 * g.ldb), 0, (int)(((int64_t)(b_rows - 1) * g.ldb + g.K) * 2), 0x00020000);
  uint32_t a_off[SA], b_off[SB];
#pragma unroll
  for (int i = 0; i < SA; ++i) a_off[i] = (uint32_t)(((int64_t)(s_row + 32 * i) * g.lda + s_kc) * ES);
#pragma unroll
  for (int i = 0; i < SB; ++i) b_off[i] = (uint32_t)(((int64_t)(s_row + 32 * i) * g.ldb + s_kc) * 2);
  u32x4 ra[SA], rb[SB];
  auto load_a = [&](uint32_t voff, int soff) -> u32x4 {
    if constexpr (ES == 2) {
      return __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, (int)voff, soff, 0);
    } else {
      const u32x4 lo = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, (int)voff, soff, 0);
      const u32x4 hi = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, (int)(voff + 16), soff, 0);
      return u32x4{cvt_pk_bf16(__uint_as_float(lo[0]), __uint_as_float(lo[1])),
                   cvt_pk_bf16(__uint_as_float(lo[2]), __uint_as_float(lo[3])),
                   cvt_pk_bf16(__uint_as_float(hi[0]), __uint_as_float(hi[1])),
                   cvt_pk_bf16(__uint_as_float(hi[2]), __uint_as_float(hi[3]))};
    }
  };
  auto fetch = [&](int k0) {
    if (k0 + BK <= g.K) {  // full stage (uniform)
#pragma unroll
      for (int i = 0; i < SA; ++i) ra[i] = load_a(a_off[i], k0 * ES);
#pragma unroll
      for (int i = 0; i < SB; ++i) rb[i] = __builtin_amdgcn_raw_buffer_load_b128(b_rsrc, (int)b_off[i], k0 * 2, 0);
    } else {               // last partial stage: chunks at k >= K are zero. k0 is added to the checked
                           // (vector) offset here, so nothing past the last row's end is touched.
      const bool k_ok = k0 + s_kc < g.K;
#pragma unroll
      for (int i = 0; i < SA; ++i) {
        const u32x4 v = load_a(a_off[i] + (uint32_t)(k0 * ES), 0);
        ra[i] = k_ok ? v : u32x4{0, 0, 0, 0};
      }
#pragma unroll
      for (int i = 0; i < SB; ++i) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(b_rsrc, (int)(b_off[i] + (uint32_t)(k0 * 2)), 0, 0);
        rb[i] = k_ok ? v : u32x4{0, 0, 0, 0};
      }
    }
  };
  auto stage = [&]() {
#pragma unroll
    for (int i = 0; i < SA; ++i) *reinterpret_cast<u32x4*>(&lds_a[(s_row + 32 * i) * kLdsRow + s_kc]) = ra[i];
#pragma unroll
    for (int i = 0; i < SB; ++i) *reinterpret_cast<u32x4*>(&lds_b[(s_row + 32 * i) * kLdsRow + s_kc]) = rb[i];
  };

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  fetch(0);
  for (int k0 = 0; k0 < g.K; k0 += BK) {
    __syncthreads();  // previous iteration's fragment reads are done
    stage();
    __syncthreads();
    if (k0 + BK < g.K) fetch(k0 + BK);
#pragma unroll
    for (int ks = 0; ks < BK; ks += 16) {
      bf16x8 fa[4], fb[2];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        fa[i] = *reinterpret_cast<const bf16x8*>(&lds_a[(wm + i * 32 + lane % 32) * kLdsRow + ks + (lane / 32) * 8]);
#pragma unroll
      for (int j = 0; j < 2; ++j)
        fb[j] = *reinterpret_cast<const bf16x8*>(&lds_b[(wn + j * 32 + lane % 32) * kLdsRow + ks + (lane / 32) * 8]);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  }

  // epilogue. 32x32 accumulator: register e of lane l is row (e/4)*8 + (l/32)*4 + e%4, column l%32.
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int n = n0 + wn + j * 32 + lane % 32;
    if (n >= gr.N) continue;
    // project: the column decides buffer, head block and rank once; the row adds b and pos
    int side = 0;
    int64_t col_off = 0, seq_stride = 0;
    int rank = 0;
    if (g.mode == kProject) {
      col_off = project_dst(g, n, 0, 0, &side);
      const int64_t one = project_dst(g, n, 0, 1, &side);
      rank = (int)(one - col_off);
      seq_stride = (int64_t)g.max_seq * (side ? g.RV : g.RK);
    }
    void* cache = side ? g.C2 : g.C;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wm + i * 32 + (e / 4) * 8 + (lane / 32) * 4 + e % 4;
        if (m >= g.M) continue;
        if (g.mode == kProject) {
          int b, pos;
          if (token_dst(g, m, &b, &pos))
            store_cache(g, cache, (int64_t)b * seq_stride + col_off + (int64_t)pos * rank, acc[i][j][e]);
        } else {
          store_out(static_cast<TC*>(g.C) + gr.c_off + (int64_t)m * g.ldc + n, acc[i][j][e]);
        }
      }
    }
  }
}

// ---- query absorption for few rows (decode: T = batch) -------------------------------------------
// q'_hq = q_hq . B_k^T has K = d_head <= 128: at most four MFMA steps. One wavefront per (query head,
// 16 latent columns) keeps the whole B operand of its tile in registers and walks the row tiles;
// with a few dozen rows this is a launch of a few hundred independent waves and no LDS.
template <typename TC>
__device__ __forceinline__ void absorb_query_small_body(const GemmArgs& g, const int col_tile, const int head,
                                                        const int lane) {
  const Group gr = group_of(g, head);
  const int n0 = col_tile * 16;
  if (n0 >= gr.N) return;
  const int ln = lane % 16, lg = lane / 16;
  const uint16_t* A = static_cast<const uint16_t*>(g.A) + gr.a_off;
  const uint16_t* B = static_cast<const uint16_t*>(g.B) + gr.b_off;
  union Fr { u32x4 u; bf16x8 v; };
  Fr b[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const int col = 32 * ks + 8 * lg;
    b[ks].u = col < g.K ? *reinterpret_cast<const u32x4*>(B + (int64_t)(n0 + ln) * g.ldb + col) : u32x4{0, 0, 0, 0};
  }
  for (int m0 = 0; m0 < g.M; m0 += 16) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int col = 32 * ks + 8 * lg;
      Fr a;
      a.u = (m0 + ln < g.M && col < g.K) ? *reinterpret_cast<const u32x4*>(A + (int64_t)(m0 + ln) * g.lda + col)
                                         : u32x4{0, 0, 0, 0};
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b[ks].v, acc, 0, 0, 0);
    }
    // register e of lane l is row 4 * (l / 16) + e, column l % 16
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int m = m0 + 4 * lg + e;
      if (m < g.M) store_out(static_cast<TC*>(g.C) + gr.c_off + (int64_t)m * g.ldc + n0 + ln, acc[e]);
    }
  }
}

template <typename TC>
__global__ __launch_bounds__(64) void absorb_query_small_kernel(const GemmArgs g) {
  absorb_query_small_body<TC>(g, blockIdx.x, blockIdx.y, threadIdx.x);
}

// ---- per-head products with many rows (prefill query absorption, the fold of B_v into W_o) -------
// K = d_head <= 128 and N = rank <= 128: 1 flop per 2 bytes, a stream over A (read once) and C
// (written once). A workgroup takes 256 rows of one head: the head's B rows (at most 128 x 128) go
// to LDS once, each of the four waves loads the A fragments of its four 16-row tiles straight from
// global memory in MFMA layout (a row's 2 K bytes are contiguous, so the four k-steps of a tile use
// whole lines) and walks the head's column tiles with a B fragment in registers shared by its four
// row tiles. The product is taken transposed (B rows first), which leaves a lane with four
// consecutive columns of one output row: one 8- or 16-byte store.
constexpr int kRowsBRow = 128 + 16;   // LDS row of the B tile: 18 chunks, conflict-free fragment reads
constexpr int kRowsPerWg = 256;

template <typename TC>
__global__ __launch_bounds__(256) void grouped_rows_kernel(const GemmArgs g) {
  __shared__ __attribute__((aligned(16))) uint16_t lds_b[128 * kRowsBRow];
  const Group gr = group_of(g, blockIdx.y);
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64, ln = lane % 16, lg = lane / 16;
  const uint16_t* A = static_cast<const uint16_t*>(g.A) + gr.a_off;
  const uint16_t* B = static_cast<const uint16_t*>(g.B) + gr.b_off;
  const int ksteps = (g.K + 31) / 32;
  // the head's B rows: N rows of K elements, K / 8 chunks of 16 bytes each; columns K .. 128 are never read
  {
    const int cpr = g.K / 8;
    for (int i = tid; i < gr.N * cpr; i += 256) {
      const int r = i / cpr, c = i - r * cpr;
      *reinterpret_cast<u32x4*>(&lds_b[r * kRowsBRow + c * 8]) = *reinterpret_cast<const u32x4*>(B + (int64_t)r * g.ldb + c * 8);
    }
  }
  // A fragments of the wave's four row tiles: lane (ln, lg) holds k = 32 ks + 8 lg .. + 8 of row ln
  const int row0 = blockIdx.x * kRowsPerWg + wave * 64;
  const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(A), 0, (int)(((int64_t)(g.M - 1) * g.lda + g.K) * 2), 0x00020000);
  union Fr { u32x4 u; bf16x8 v; };
  Fr af[4][4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int row = row0 + 16 * t + ln, col = 32 * ks + 8 * lg;
      af[t][ks].u = __builtin_amdgcn_raw_buffer_load_b128(
          a_rsrc, (int)((row < g.M && col < g.K) ? (uint32_t)(((int64_t)row * g.lda + col) * 2) : 0x80000000u), 0, 2);
    }
  __syncthreads();
  TC* C = static_cast<TC*>(g.C) + gr.c_off;
  for (int n0 = 0; n0 < gr.N; n0 += 16) {
    f32x4 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if (ks >= ksteps) break;
      Fr b;
      const int col = 32 * ks + 8 * lg;
      b.u = col < g.K ? *reinterpret_cast<const u32x4*>(&lds_b[(n0 + ln) * kRowsBRow + col]) : u32x4{0, 0, 0, 0};
#pragma unroll
      for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b.v, af[t][ks].v, acc[t], 0, 0, 0);
    }
    // register e of lane l: column n0 + 4 * (l / 16) + e of row l % 16
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int row = row0 + 16 * t + ln;
      if (row >= g.M) continue;
      TC* dst = C + (int64_t)row * g.ldc + n0 + 4 * lg;
      if constexpr (sizeof(TC) == 4) {
        *reinterpret_cast<f32x4*>(dst) = acc[t];
      } else {
        uint2 w;
        w.x = cvt_pk_bf16(acc[t][0], acc[t][1]);
        w.y = cvt_pk_bf16(acc[t][2], acc[t][3]);
        *reinterpret_cast<uint2*>(dst) = w;
      }
    }
  }
}

// ---- bf16 MFMA kernel for the large products (prefill: M = tokens of the batch) ----------------
// Workgroup tile 256 x 256, k stage 64, eight waves in a 2 x 4 grid, each wave 128 x 64 as 4 x 2
// v_mfma_f32_32x32x16_bf16 tiles. Both operands go from global memory straight into LDS
// (buffer_load ... lds, 16 bytes per lane), two stages of 64 KiB in a ring: while stage t is
// multiplied, stage t+1 is in flight, and stage t+2 is requested as soon as every wave has read the
// last fragment of stage t. A wave-wide load fills 1 KiB of LDS in lane order, so the padding that
// keeps fragment reads conflict free is replaced by a swizzle: tile row r keeps its 16-byte chunk c
// at position c ^ ((r / 2) % 8) of its 128-byte LDS row, which the loading lane applies to its
// global address and the reading lane to its LDS address. Rows past M / N and the k tail are
// zero-filled by the buffer range check (their offsets are forced out of range), so the loop has
// no conditional loads. The loads are issued through inline assembly: the compiler then keeps no
// dependency between them and the LDS reads, and the kernel orders the two itself with vmcnt waits
// in front of its barriers.
// The chip is power limited on this kernel (the shader clock falls from 2.4 to about 1.3-1.5 GHz
// while it runs), so what counts is work per byte moved: the 256 x 256 tile halves the L2 -> LDS
// traffic per flop of a 256 x 128 tile, and the epilogue writes full 128-byte lines.
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
constexpr int DM = 256, DN = 256, DK = 64;
constexpr int kDmaStage = (DM + DN) * DK;     // elements per ring stage (A rows, then B rows)

__device__ __forceinline__ void dma16(i32x4 rsrc, uint32_t lds_addr, uint32_t voff, int soff) {
  // lane l of the wave lands at lds_addr + 16 * l
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :: "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory", "m0");
}
__device__ __forceinline__ i32x4 make_rsrc(const void* p, uint32_t bytes) {
  const uint64_t a = (uint64_t)p;
  return i32x4{__builtin_amdgcn_readfirstlane((int)(uint32_t)a), __builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32)),
               __builtin_amdgcn_readfirstlane((int)bytes), 0x00020000};
}
__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
constexpr int vm_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x70 | 0xF00; }  // s_waitcnt vmcnt(n) only

// One TM x TN tile of C at (m0, n0). The eight waves form a WMW x WNW grid:
//   256 x 256, 2 x 4 waves of 128 x 64: the full tile;
//   256 x 64,  8 x 1 waves of 32 x 64: a column tile with at most 64 valid columns (the ragged last column
//              tile of an N that is not a multiple of 256 costs a quarter of the multiplies);
//   128 x 256, 2 x 4 waves of 64 x 64: half a full tile, for the tiles of an incomplete last round of the
//              launch (see the kernel).
template <typename TC, int WMW, int WNW, int TM, int TN>
__device__ __forceinline__ void dma_tile(const GemmArgs& g, const int m0, const int n0, uint16_t* lds) {
  static_assert(WMW * WNW == 8 && TM % 64 == 0 && TN % 64 == 0, "eight waves, load rounds of 64 rows");
  constexpr int WM = TM / WMW, CW = TN / WNW;    // rows and columns of a wave's tile
  constexpr int IB = WM / 32, FB = CW / 32;      // 32 x 32 blocks of it
  constexpr int LA = TM / 64, LB = TN / 64;      // wave-wide load rounds of the A rows and the B rows
  constexpr int LQ = LA + LB;                    // loads per wave and stage
  constexpr int kStage = (TM + TN) * DK;         // elements per ring stage (A rows, then B rows)
  const int M = g.M, N = g.N, K = g.K;

  const int tid = threadIdx.x, lane = tid % 64;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const int wm = (wave / WNW) * WM, wn = (wave % WNW) * CW;
  const uint16_t* A = static_cast<const uint16_t*>(g.A);
  const uint16_t* B = static_cast<const uint16_t*>(g.B);
  const int a_rows = min(TM, M - m0), b_rows = min(TN, N - n0);
  const i32x4 a_rsrc = make_rsrc(A + (int64_t)m0 * g.lda, (uint32_t)(((int64_t)(a_rows - 1) * g.lda + K) * 2));
  const i32x4 b_rsrc = make_rsrc(B + (int64_t)n0 * g.ldb, (uint32_t)(((int64_t)(b_rows - 1) * g.ldb + K) * 2));

  // the lane's source in a wave-wide load: tile row lane / 8 of the wave's 8 rows, LDS chunk lane % 8
  const int l_row = wave * 8 + lane / 8;
  const int l_chunk = (lane % 8) ^ ((l_row / 2) % 8);
  constexpr uint32_t kOob = 0x80000000u;
  const int nk = (K + DK - 1) / DK;
  const int k_tail0 = (nk - 1) * DK;
  const bool has_tail = (K % DK) != 0;
  const bool tail_ok = k_tail0 + l_chunk * 8 < K;
  uint32_t a_off[4], b_off[4], a_tail[4], b_tail[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = j * 64 + l_row;
    a_off[j] = row < a_rows ? (uint32_t)(((int64_t)row * g.lda + l_chunk * 8) * 2) : kOob;
    b_off[j] = row < b_rows ? (uint32_t)(((int64_t)row * g.ldb + l_chunk * 8) * 2) : kOob;
    // the tail stage carries k0 in the range-checked offset, so nothing past a row's end is read
    a_tail[j] = (row < a_rows && tail_ok) ? a_off[j] + (uint32_t)(k_tail0 * 2) : kOob;
    b_tail[j] = (row < b_rows && tail_ok) ? b_off[j] + (uint32_t)(k_tail0 * 2) : kOob;
  }
  const uint32_t lds0 = lds_addr_of(lds) + (uint32_t)(wave * 8 * DK * 2);
  // load q (0..LA-1: A rows, LA..: B rows) of stage t into ring buffer s
  auto issue1 = [&](int s, int t, int q) {
    const bool is_a = q < LA;
    const int j = is_a ? q : q - LA;
    const uint32_t dst = lds0 + (uint32_t)((s * kStage + (is_a ? 0 : TM * DK) + j * 64 * DK) * 2);
    const bool tail = has_tail && t == nk - 1;
    const uint32_t voff = is_a ? (tail ? a_tail[j] : a_off[j]) : (tail ? b_tail[j] : b_off[j]);
    dma16(is_a ? a_rsrc : b_rsrc, dst, voff, tail ? 0 : t * DK * 2);
  };

  // fragment addressing: row lane % 32 of a 32-row block, chunk 2 * kstep + lane / 32
  const int f_row = lane % 32;
  int f_off[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) f_off[s] = f_row * DK + (((2 * s + lane / 32) ^ ((f_row / 2) % 8)) * 8);

  f32x16 acc[IB][FB];
#pragma unroll
  for (int i = 0; i < IB; ++i)
#pragma unroll
    for (int j = 0; j < FB; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  bf16x8 fa0[IB], fb0[FB], fa1[IB], fb1[FB];
  auto load_frag = [&](int s, int ks, bf16x8 (&fa)[IB], bf16x8 (&fb)[FB]) {
    const uint16_t* sa = lds + s * kStage + wm * DK;
    const uint16_t* sb = lds + s * kStage + TM * DK + wn * DK;
#pragma unroll
    for (int i = 0; i < IB; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(&sa[i * 32 * DK + f_off[ks]]);
#pragma unroll
    for (int j = 0; j < FB; ++j) fb[j] = *reinterpret_cast<const bf16x8*>(&sb[j * 32 * DK + f_off[ks]]);
  };
  // operands swapped: the accumulator tile is C^T, a lane holds one m and runs of four n
  auto mma = [&](bf16x8 (&fa)[IB], bf16x8 (&fb)[FB]) {
#pragma unroll
    for (int i = 0; i < IB; ++i)
#pragma unroll
      for (int j = 0; j < FB; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
  };
  constexpr int kVm0Lgkm0 = 0x0070;   // s_waitcnt vmcnt(0) lgkmcnt(0)

  // Stage t in ring buffer s; fragments of its k step 0 are in fa0/fb0 on entry. Straight-line
  // (the last stage reads the other buffer into registers nobody uses) so that the compiler's wait
  // counters see one path and leave the reads in flight across the multiplies. The scheduling
  // barriers pin "reads of the next k step first, then the multiplies that hide them".
  auto step = [&](int s, int t) {
    load_frag(s, 1, fa1, fb1);
    __builtin_amdgcn_sched_barrier(0);
    mma(fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    load_frag(s, 2, fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    mma(fa1, fb1);
    __builtin_amdgcn_sched_barrier(0);
    load_frag(s, 3, fa1, fb1);
    __builtin_amdgcn_sched_barrier(0);
    mma(fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    // this wave's reads of stage t have returned and its part of stage t+1 has landed; after the
    // barrier that holds for every wave and buffer s can be refilled with stage t+2
    __builtin_amdgcn_s_waitcnt(kVm0Lgkm0);
    asm volatile("s_barrier" ::: "memory");
    load_frag(1 - s, 0, fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    const bool more = t + 2 < nk;
#pragma unroll
    for (int i = 0; i < IB; ++i)
#pragma unroll
      for (int j = 0; j < FB; ++j) {   // the loads of stage t+2 go between the last multiplies, one each
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb1[j], fa1[i], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (more && i * FB + j < LQ) issue1(s, t + 2, i * FB + j);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
    for (int q = IB * FB; q < LQ; ++q)   // a narrow tile has fewer multiplies than loads
      if (more) issue1(s, t + 2, q);
  };

#pragma unroll
  for (int q = 0; q < LQ; ++q) issue1(0, 0, q);
  if (1 < nk) {
#pragma unroll
    for (int q = 0; q < LQ; ++q) issue1(1, 1, q);
    __builtin_amdgcn_s_waitcnt(vm_imm(LQ));
  } else {
    __builtin_amdgcn_s_waitcnt(vm_imm(0));
  }
  asm volatile("s_barrier" ::: "memory");
  load_frag(0, 0, fa0, fb0);
  const int pairs = (nk - 1) / 2;   // pairs of stages in which every stage has a successor
  int t = 0;
  for (int p = 0; p < pairs; ++p, t += 2) {
    step(0, t);
    step(1, t + 1);
  }
  step(0, t);
  if (nk - t > 1) step(1, t + 1);

  // Epilogue. Accumulator (i, j): register e of lane l is n = wn + j*32 + (e/4)*8 + (l/32)*4 + e%4,
  // m = wm + i*32 + l%32.
  if constexpr (sizeof(TC) == 4) {
    // fp32 C (plain mode only): 16 bytes per lane straight from the registers
#pragma unroll
    for (int i = 0; i < IB; ++i) {
      const int m = m0 + wm + i * 32 + lane % 32;
      if (m >= M) continue;
      float* crow = static_cast<float*>(g.C) + (int64_t)m * g.ldc;
#pragma unroll
      for (int j = 0; j < FB; ++j)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const int n = n0 + wn + j * 32 + gq * 8 + (lane / 32) * 4;
          if (n + 3 < N && g.ldc % 4 == 0) {
            *reinterpret_cast<float4*>(crow + n) = float4{acc[i][j][gq * 4], acc[i][j][gq * 4 + 1], acc[i][j][gq * 4 + 2], acc[i][j][gq * 4 + 3]};
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) if (n + e < N) crow[n + e] = acc[i][j][gq * 4 + e];
          }
        }
    }
  } else {
    // bf16 C: each wave turns 64 of its rows (32 in a narrow tile) at a time into bf16 in a private LDS region (row
    // stride 144 bytes) and streams them out as 16-byte chunks; 8 lanes cover one 128-byte row of
    // the wave's tile, so a store instruction writes 8 full lines (plain) or 8 runs of 128 bytes
    // of one token's latent rows (project).
    asm volatile("s_barrier" ::: "memory");   // every wave is done with the last stage
    constexpr int EROW = 72;
    constexpr int GB = IB < 2 ? IB : 2;   // 32-row blocks per round
    uint16_t* ep = lds + wave * (64 * EROW);
    const int c = lane % 8;
    const int n = n0 + wn + c * 8;
    int side = 0, rank = 0;
    int64_t col_off = 0, seq_stride = 0;
    if (g.mode == kProject && n < N) {   // the 8 columns of a chunk lie in one head: ranks are multiples of 16
      col_off = project_dst(g, n, 0, 0, &side);
      rank = (int)(project_dst(g, n, 0, 1, &side) - col_off);
      seq_stride = (int64_t)g.max_seq * (side ? g.RV : g.RK);
    }
    uint16_t* cbase = static_cast<uint16_t*>((g.mode == kProject && side) ? g.C2 : g.C);
    const bool wide = g.mode == kProject || g.ldc % 8 == 0;
    if (g.mode == kProject && g.cache_fp8) {
      // E4M3 cache: the same transposition with one byte per element. Four accumulators become four
      // codes (saturated, rounded from the fp32 value) in one LDS word; a lane then scatters the eight
      // codes of its chunk with one 8-byte store.
      uint8_t* ep8 = reinterpret_cast<uint8_t*>(ep);
      uint8_t* cb8 = reinterpret_cast<uint8_t*>(cbase);
      auto sat = [](float v) { return fminf(fmaxf(v, -448.f), 448.f); };
#pragma unroll
      for (int h = 0; h < IB / GB; ++h) {
#pragma unroll
        for (int ii = 0; ii < GB; ++ii)
#pragma unroll
          for (int j = 0; j < FB; ++j)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
              const int i = GB * h + ii;
              uint32_t w = __builtin_amdgcn_cvt_pk_fp8_f32(sat(acc[i][j][gq * 4 + 0]), sat(acc[i][j][gq * 4 + 1]), 0u, false);
              w = __builtin_amdgcn_cvt_pk_fp8_f32(sat(acc[i][j][gq * 4 + 2]), sat(acc[i][j][gq * 4 + 3]), w, true);
              *reinterpret_cast<uint32_t*>(&ep8[(ii * 32 + lane % 32) * EROW + j * 32 + gq * 8 + (lane / 32) * 4]) = w;
            }
#pragma unroll
        for (int it = 0; it < 4 * GB; ++it) {
          const int row = it * 8 + lane / 8;
          const int m = m0 + wm + h * 32 * GB + row;
          const uint2 v = *reinterpret_cast<const uint2*>(&ep8[row * EROW + c * 8]);
          if (m >= M || n >= N) continue;
          int b, pos;
          if (!token_dst(g, m, &b, &pos)) continue;
          *reinterpret_cast<uint2*>(cb8 + (int64_t)b * seq_stride + col_off + (int64_t)pos * rank) = v;
        }
      }
      return;
    }
#pragma unroll
    for (int h = 0; h < IB / GB; ++h) {
#pragma unroll
      for (int ii = 0; ii < GB; ++ii)
#pragma unroll
        for (int j = 0; j < FB; ++j)
#pragma unroll
          for (int gq = 0; gq < 4; ++gq) {
            const int i = GB * h + ii;
            uint2 v;
            v.x = cvt_pk_bf16(acc[i][j][gq * 4 + 0], acc[i][j][gq * 4 + 1]);
            v.y = cvt_pk_bf16(acc[i][j][gq * 4 + 2], acc[i][j][gq * 4 + 3]);
            *reinterpret_cast<uint2*>(&ep[(ii * 32 + lane % 32) * EROW + j * 32 + gq * 8 + (lane / 32) * 4]) = v;
          }
#pragma unroll
      for (int it = 0; it < 4 * GB; ++it) {
        const int row = it * 8 + lane / 8;
        const int m = m0 + wm + h * 32 * GB + row;
        const u32x4 v = *reinterpret_cast<const u32x4*>(&ep[row * EROW + c * 8]);
        if (m >= M || n >= N) continue;
        int b = 0, pos = 0;
        if (g.mode == kProject && !token_dst(g, m, &b, &pos)) continue;
        uint16_t* dst = g.mode == kProject ? cbase + (int64_t)b * seq_stride + col_off + (int64_t)pos * rank
                                           : cbase + (int64_t)m * g.ldc + n;
        if (n + 7 < N && wide) {
          *reinterpret_cast<u32x4*>(dst) = v;
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (n + e < N) dst[e] = (uint16_t)(v[e / 2] >> (16 * (e % 2)));
        }
      }
    }
  }
}

template <typename TC>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void gemm_dma_kernel(const GemmArgs g) {
  __shared__ __attribute__((aligned(1024))) uint16_t lds[2 * kDmaStage];
  // A compute unit holds one workgroup, so a launch runs in rounds of as many tiles as there are compute
  // units. When the last round is at most half full, its tiles are cut into two 128-row halves (blocks from
  // g.split_from on, two per tile): the round then takes about half a tile's time instead of a whole one.
  int slot = blockIdx.x, half = -1;
  if (slot >= g.split_from) {
    half = (slot - g.split_from) & 1;
    slot = g.split_from + (slot - g.split_from) / 2;
  }
  // tile order: XCD-major, then 8 row tiles down before the next column tile (see gemm_bf16_kernel)
  const int mt = (g.M + DM - 1) / DM, nt = g.nt;
  const int tiles = mt * nt, per_xcd = (tiles + 7) / 8;
  const int lin = (slot % 8) * per_xcd + slot / 8;
  if (lin >= tiles) return;
  constexpr int GM = 8;
  const int band = lin / (GM * nt), in_band = lin % (GM * nt);
  const int band_rows = min(GM, mt - band * GM);
  const int tm = band * GM + in_band % band_rows, tn = in_band / band_rows;
  const int m0 = tm * DM, n0 = tn * DN;
  if (g.N - n0 <= 64) {
    if (half <= 0) dma_tile<TC, 8, 1, DM, 64>(g, m0, n0, lds);   // cheap already: not cut, the second block has nothing to do
  } else if (half < 0) {
    dma_tile<TC, 2, 4, DM, DN>(g, m0, n0, lds);
  } else if (m0 + half * (DM / 2) < g.M) {
    dma_tile<TC, 2, 4, DM / 2, DN>(g, m0 + half * (DM / 2), n0, lds);
  }
}

// ---- bf16 MFMA kernel for few rows (decode: M = batch) ------------------------------------------
// With M <= 64 the product is a weight stream: every B row (K contiguous bf16) is read once and
// the kernel is bound by HBM, not by MFMA. A workgroup of eight waves owns 16 rows of B; the
// waves split K into eight contiguous ranges, so a launch has ceil(N/16) * 8 waves in flight
// (about 1500 to 2000 at the 7B shapes) instead of the few 128 x 128 tiles of the large kernel.
// Each wave accumulates MT 16 x 16 tiles (v_mfma_f32_16x16x32_bf16), the eight partial tiles are
// summed through LDS in a fixed order (deterministic) and written by one wave per row tile.
constexpr int kSkinnyWaves = 8;

constexpr int kSkinnyChunkK = 512;             // k covered by one wave-wide 16-byte-per-lane load of a row
// Padded LDS row (elements): 66 chunks of 16 bytes. The MFMA fragment read (lane (ln, lg): row ln,
// chunk lg) is free of bank conflicts when the row stride is 2 (mod 16) chunks, because the LDS
// serves eight lanes of lane row lg and eight of lane row lg + 1 in one pass (measured); the stride
// of 1 (mod 16) that suits lane-row passes gave a two-way conflict on every read.
constexpr int kSkinnyRow = kSkinnyChunkK + 16;

template <typename TA, typename TC, int MT>
__global__ __launch_bounds__(kSkinnyWaves * 64) void gemm_skinny_kernel(const GemmArgs g) {
  // per wave: 16 weight rows x 512 k, staged so that global reads are 1 KiB contiguous per row
  // (HBM-friendly) while the MFMA operand wants 16 rows x 64 bytes per instruction
  extern __shared__ __attribute__((aligned(16))) uint16_t skinny_lds[];
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int ln = lane % 16, lg = lane / 16;
  const int n0 = blockIdx.x * 16;
  const TA* A = static_cast<const TA*>(g.A);
  const uint16_t* B = static_cast<const uint16_t*>(g.B);
  uint16_t* wl = skinny_lds + wave * 16 * kSkinnyRow;
  const int k_per_wave = ((g.K + kSkinnyWaves - 1) / kSkinnyWaves + 31) / 32 * 32;
  const int k_begin = wave * k_per_wave, k_end = min(g.K, k_begin + k_per_wave);
  f32x4 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  // Every load below is unconditional: the raw-buffer range check returns zeros for rows past N / M
  // (their offsets are forced out of range) and a guarded load would cost a branch and a wait each.
  const int b_rows = min(16, g.N - n0);
  const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(B + (int64_t)n0 * g.ldb), 0, (int)(((int64_t)(b_rows - 1) * g.ldb + g.K) * 2), 0x00020000);
  constexpr int ES = (int)sizeof(TA);
  const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<TA*>(A), 0, (int)(((int64_t)(g.M - 1) * g.lda + g.K) * ES), 0x00020000);
  uint32_t a_row[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
    a_row[mt] = 16 * mt + ln < g.M ? (uint32_t)((int64_t)(16 * mt + ln) * g.lda * ES) : 0x80000000u;
  auto load_a = [&](uint32_t voff) -> u32x4 {
    if constexpr (ES == 2) {
      return __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, (int)voff, 0, 0);
    } else {
      const u32x4 lo = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, (int)voff, 0, 0);
      const u32x4 hi = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, (int)(voff + 16), 0, 0);
      return u32x4{cvt_pk_bf16(__uint_as_float(lo[0]), __uint_as_float(lo[1])),
                   cvt_pk_bf16(__uint_as_float(lo[2]), __uint_as_float(lo[3])),
                   cvt_pk_bf16(__uint_as_float(hi[0]), __uint_as_float(hi[1])),
                   cvt_pk_bf16(__uint_as_float(hi[2]), __uint_as_float(hi[3]))};
    }
  };
  constexpr int SG = 16 / MT;  // MFMA steps whose A chunks are requested together
  for (int kc = k_begin; kc < k_end; kc += kSkinnyChunkK) {
    // 1. sixteen row loads in flight, each 1 KiB contiguous across the wave
    u32x4 rows[16];
    const uint32_t k_lane = (uint32_t)(kc + lane * 8);
#pragma unroll
    for (int i = 0; i < 16; ++i)
      rows[i] = __builtin_amdgcn_raw_buffer_load_b128(
          b_rsrc, (int)(i < b_rows ? (uint32_t)(((int64_t)i * g.ldb + k_lane) * 2) : 0x80000000u), 0, 2);
    // 2. MFMA steps of 32 k: B operand from the wave's LDS strip, A operand (few rows, cache resident)
    //    from global, SG steps requested at a time. Chunks at k >= K are zeroed in A (the B strip may
    //    hold the neighbouring range there). The first group of A chunks is requested before the B
    //    rows are waited for, so the two latencies overlap.
    const int steps = (min(kSkinnyChunkK, k_end - kc) + 31) / 32;
    u32x4 fa[SG][MT];
    auto request_a = [&](int s0) {
#pragma unroll
      for (int u = 0; u < SG; ++u) {
        const int k = kc + 32 * (s0 + u) + 8 * lg;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const u32x4 v = load_a(k < g.K ? a_row[mt] + (uint32_t)(k * ES) : 0x80000000u);
          fa[u][mt] = v;
        }
      }
    };
    request_a(0);
#pragma unroll
    for (int i = 0; i < 16; ++i) *reinterpret_cast<u32x4*>(&wl[i * kSkinnyRow + lane * 8]) = rows[i];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (int s0 = 0; s0 < steps; s0 += SG) {
      if (s0 > 0) request_a(s0);
#pragma unroll
      for (int u = 0; u < SG; ++u) {
        if (s0 + u >= steps) break;
        union { u32x4 u4; bf16x8 v; } b;
        b.u4 = *reinterpret_cast<const u32x4*>(&wl[ln * kSkinnyRow + 32 * (s0 + u) + 8 * lg]);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          union { u32x4 u4; bf16x8 v; } a;
          a.u4 = fa[u][mt];
          acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, acc[mt], 0, 0, 0);
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  // 3. sum the eight k ranges through LDS in a fixed order; the strip is reused as [wave][mt][lane] f32x4
  __syncthreads();
  f32x4* red = reinterpret_cast<f32x4*>(skinny_lds);
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) red[(wave * MT + mt) * 64 + lane] = acc[mt];
  __syncthreads();
  if (wave < MT) {  // wave w finishes row tile w. Register e of lane l is row 4 * (l / 16) + e, column l % 16.
    f32x4 sum = red[wave * 64 + lane];
#pragma unroll
    for (int w = 1; w < kSkinnyWaves; ++w) sum += red[(w * MT + wave) * 64 + lane];
    const int n = n0 + ln;
    if (n < g.N) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int m = 16 * wave + 4 * lg + e;
        if (m >= g.M) continue;
        if (g.mode == kProject) {
          int side, b, pos;
          if (!token_dst(g, m, &b, &pos)) continue;
          const int64_t dst = project_dst(g, n, b, pos, &side);
          store_cache(g, side ? g.C2 : g.C, dst, sum[e]);
        } else {
          store_out(static_cast<TC*>(g.C) + (int64_t)m * g.ldc + n, sum[e]);
        }
      }
    }
  }
}

constexpr size_t kSkinnyLdsBytes = (size_t)kSkinnyWaves * 16 * kSkinnyRow * sizeof(uint16_t);  // 135168

template <typename TA, typename TC>
static void launch_skinny(const GemmArgs& a, hipStream_t st) {
  const dim3 grid((a.N + 15) / 16), block(kSkinnyWaves * 64);
  const int mt = (a.M + 15) / 16;
  auto go = [&](auto kern) {
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(kern), kSkinnyLdsBytes) != hipSuccess) return;
    hipLaunchKernelGGL(kern, grid, block, kSkinnyLdsBytes, st, a);
  };
  if (mt == 1) go(gemm_skinny_kernel<TA, TC, 1>);
  else if (mt == 2) go(gemm_skinny_kernel<TA, TC, 2>);
  else if (mt == 3) go(gemm_skinny_kernel<TA, TC, 3>);
  else go(gemm_skinny_kernel<TA, TC, 4>);
}

// ---- the same weight stream at M <= 16 (one MFMA row tile: the decode batch) ---------------------
// Timing stamps inside the kernel above showed what bounds a launch this short (27 MB of weights is
// ~0.1 MB per compute unit): each compute unit pulls its bytes through one vector-memory pipe, and the
// activations (16 x K, read again by every workgroup, from L2) load that pipe as much as the weights.
// So here (a) every load of a chunk, activations and weights, is in flight before the first wait,
// (b) the activations are requested first and read like the weights (1 KiB contiguous per
// instruction: half the requests of 64-byte fragment reads): they come from L2, land early, and
// are transposed through the wave's LDS strip while the weight rows are still on their way from
// HBM; fp32 activations are rounded to bf16 at that point, (c) the sixteen LDS fragment reads of
// the weights are issued together instead of one wait per MFMA. WAVES waves split K.
template <typename TA, typename TC, int WAVES>
__device__ __forceinline__ void skinny16_body(const GemmArgs& g, const int col_tile, uint16_t* skinny_lds) {
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int ln = lane % 16, lg = lane / 16;
  const int n0 = col_tile * 16;
  const uint16_t* B = static_cast<const uint16_t*>(g.B);
  uint16_t* wl = skinny_lds + wave * 16 * kSkinnyRow;
  const int k_per_wave = ((g.K + WAVES - 1) / WAVES + 63) / 64 * 64;
  const int k_begin = wave * k_per_wave, k_end = min(g.K, k_begin + k_per_wave);
  f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
  // unconditional loads: offsets of rows past N / M and of k past the wave's range are forced out of
  // the buffer's range and return zeros
  const int b_rows = min(16, g.N - n0);
  constexpr int ES = (int)sizeof(TA);
  const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(B + (int64_t)n0 * g.ldb), 0, (int)(((int64_t)(b_rows - 1) * g.ldb + g.K) * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(g.A), 0, (int)(((int64_t)(g.M - 1) * g.lda + g.K) * ES), 0x00020000);
  constexpr uint32_t kOut = 0x80000000u;
  auto wave_sync = [] {  // LDS writes of this wave are visible to its own later reads
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
  for (int kc = k_begin; kc < k_end; kc += kSkinnyChunkK) {
    u32x4 rows[16], fa[16], fb[16];
    [[maybe_unused]] u32x4 a_hi[ES == 4 ? 16 : 1];
    const int k_lane = kc + lane * 8;  // the lane's eight consecutive k of every row
    const uint32_t k_in = k_lane < k_end ? 0u : kOut;
    // fp32 rows are two 16-byte loads; they are rounded to bf16 only after every load of the chunk
    // has been issued (a conversion between the loads would wait for its operand and hold back the
    // loads behind it)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint32_t off = i < g.M ? k_in + (uint32_t)(((int64_t)i * g.lda + k_lane) * ES) : kOut;
      fa[i] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, (int)off, 0, 0);
      if constexpr (ES == 4) a_hi[i] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, (int)(off + 16), 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i)
      rows[i] = __builtin_amdgcn_raw_buffer_load_b128(
          b_rsrc, (int)(i < b_rows ? k_in + (uint32_t)(((int64_t)i * g.ldb + k_lane) * 2) : kOut), 0, 2);
    __builtin_amdgcn_sched_barrier(0);
    // activations: strip rows -> MFMA fragments (lane (ln, lg) holds row ln, k = 32 u + 8 lg ..)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      u32x4 v = fa[i];
      if constexpr (ES == 4)
        v = u32x4{cvt_pk_bf16(__uint_as_float(fa[i][0]), __uint_as_float(fa[i][1])),
                  cvt_pk_bf16(__uint_as_float(fa[i][2]), __uint_as_float(fa[i][3])),
                  cvt_pk_bf16(__uint_as_float(a_hi[i][0]), __uint_as_float(a_hi[i][1])),
                  cvt_pk_bf16(__uint_as_float(a_hi[i][2]), __uint_as_float(a_hi[i][3]))};
      *reinterpret_cast<u32x4*>(&wl[i * kSkinnyRow + lane * 8]) = v;
    }
    wave_sync();
#pragma unroll
    for (int u = 0; u < 16; ++u) fa[u] = *reinterpret_cast<const u32x4*>(&wl[ln * kSkinnyRow + 32 * u + 8 * lg]);
    wave_sync();
    __builtin_amdgcn_sched_barrier(0);
    // weights, the same way, as they land
#pragma unroll
    for (int i = 0; i < 16; ++i) *reinterpret_cast<u32x4*>(&wl[i * kSkinnyRow + lane * 8]) = rows[i];
    wave_sync();
#pragma unroll
    for (int u = 0; u < 16; ++u) fb[u] = *reinterpret_cast<const u32x4*>(&wl[ln * kSkinnyRow + 32 * u + 8 * lg]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      union { u32x4 u4; bf16x8 v; } a, b;
      a.u4 = fa[u], b.u4 = fb[u];
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, acc, 0, 0, 0);
    }
    wave_sync();
  }
  // sum the k ranges through LDS in a fixed order; wave 0 writes the tile
  __syncthreads();
  f32x4* red = reinterpret_cast<f32x4*>(skinny_lds);
  red[wave * 64 + lane] = acc;
  __syncthreads();
  if (wave == 0) {  // register e of lane l is row 4 * (l / 16) + e, column l % 16
    f32x4 sum = red[lane];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) sum += red[w * 64 + lane];
    const int n = n0 + ln;
    if (n < g.N) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int m = 4 * lg + e;
        if (m >= g.M) continue;
        if (g.mode == kProject) {
          int side, b, pos;
          if (!token_dst(g, m, &b, &pos)) continue;
          const int64_t dst = project_dst(g, n, b, pos, &side);
          store_cache(g, side ? g.C2 : g.C, dst, sum[e]);
        } else {
          store_out(static_cast<TC*>(g.C) + (int64_t)m * g.ldc + n, sum[e]);
        }
      }
    }
  }
}

template <typename TA, typename TC, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void gemm_skinny16_kernel(const GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) uint16_t skinny_lds[];
  skinny16_body<TA, TC, WAVES>(g, blockIdx.x, skinny_lds);
}

// The two calls that start a decode layer, K'/V' of the new tokens and the absorbed queries, do not
// depend on each other, and at decode batch each is a launch of a few microseconds that leaves
// compute units idle (the projection has N / 16 workgroups, fewer than compute units at the 7B
// shape). One launch runs both: the first n_proj workgroups are the projection's, the wavefronts of
// the rest each take one (query head, 16 latent columns) job of the query absorption.
template <typename TC, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void decode_prologue_kernel(const GemmArgs proj, const GemmArgs absq,
                                                                      const int n_proj, const int absq_col_tiles) {
  extern __shared__ __attribute__((aligned(16))) uint16_t skinny_lds[];
  if ((int)blockIdx.x < n_proj) {
    skinny16_body<uint16_t, uint16_t, WAVES>(proj, blockIdx.x, skinny_lds);
  } else {
    const int job = ((int)blockIdx.x - n_proj) * WAVES + (int)(threadIdx.x / 64);
    const int head = job / absq_col_tiles;
    if (head < absq.H * absq.G) absorb_query_small_body<TC>(absq, job % absq_col_tiles, head, threadIdx.x % 64);
  }
}

template <typename TA, typename TC>
static void launch_skinny16(const GemmArgs& a, hipStream_t st) {
  const dim3 grid((a.N + 15) / 16);
  auto go = [&](auto kern, int waves) {
    const size_t lds = (size_t)waves * 16 * kSkinnyRow * sizeof(uint16_t);
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds) != hipSuccess) return;
    hipLaunchKernelGGL(kern, grid, dim3(waves * 64), lds, st, a);
  };
  // measured at the 7B shapes (K = 4096 and K = 1100 .. 2000): eight waves pay off above 2048 k
  if (a.K > 2048) go(gemm_skinny16_kernel<TA, TC, 8>, 8);
  else go(gemm_skinny16_kernel<TA, TC, 4>, 4);
}

// ---- post-RoPE compression (Section 5.1: RoPE, then the rotation R truncated to r_h columns) ----
// One workgroup = 128 token rows and a run of kRopeHeads heads, laid out like grouped_rows_kernel: a wave
// loads the rows of its two 16-row tiles straight into MFMA fragments, and a lane's eight consecutive k
// are four RoPE pairs (2i, 2i+1), so the rotation is done in the lane's registers in fp32 and the result
// rounded to bf16 is the operand. The angles (the caller's cos / sin tables at the row's position) depend
// on the row, not on the head: a lane reads its 64 table values once and keeps them in registers for all
// heads of the workgroup (read per head they were two thirds of the kernel's vector-memory instructions
// and a third of its time). Per head the rotation's R_t rows (r_h x d_head, K = d_head <= 128) are staged
// in LDS. The product is taken transposed: a lane ends up with four consecutive latent columns of one
// token, stored at once. Queries go to q_lat, keys into the K' cache (bf16 or E4M3 codes).
constexpr int kRopeRows = 128;
constexpr int kRopeHeads = 4;

// Four waves per SIMD: the keys instantiation would take 134 registers and drop to three (64 -> 57 us with
// five registers spilled instead).
template <typename TC, bool KEYS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void rope_compress_kernel(const GemmArgs g) {
  __shared__ __attribute__((aligned(16))) uint16_t lds_b[128 * kRowsBRow];
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int ln = lane % 16, lg = lane / 16;
  const int half = g.d_head / 2;
  const int n_heads = KEYS ? g.H : g.H * g.G;   // heads of the input rows
  const int row0 = blockIdx.x * kRopeRows + wave * 32;
  const int ksteps = (g.d_head + 31) / 32;
  // the angles of the lane's rows and columns
  float4 cs[2][4], sn[2][4];
  int tok[2];
  int64_t tok_dst[2];   // keys: element offset of the token's rows in the cache, without the head's part
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int row = row0 + 16 * t + ln;
    const bool row_on = row < g.M;
    tok[t] = row_on ? row : -1;
    const int pos_raw = row_on ? g.tok_pos[row] : 0;
    const int pos = min(max(pos_raw, 0), g.n_pos - 1);
    tok_dst[t] = 0;
    if (row_on && (unsigned)pos_raw >= (unsigned)g.n_pos) {   // no angle for this position: the row is dropped
      if (g.fault) atomicOr(g.fault, kFaultPos);
      tok[t] = -1;
    } else if (KEYS && row_on) {   // keys go into the cache: a row with a bad sequence or position is dropped
      int b, pc;
      if (token_dst(g, row, &b, &pc)) tok_dst[t] = (int64_t)b * g.max_seq * g.RK;
      else tok[t] = -1;
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int col = 32 * ks + 8 * lg;
      if (row_on && col < g.d_head) {
        cs[t][ks] = *reinterpret_cast<const float4*>(g.rope_cos + (int64_t)pos * half + col / 2);
        sn[t][ks] = *reinterpret_cast<const float4*>(g.rope_sin + (int64_t)pos * half + col / 2);
      } else {
        cs[t][ks] = float4{0.f, 0.f, 0.f, 0.f}, sn[t][ks] = float4{0.f, 0.f, 0.f, 0.f};
      }
    }
  }
  union Fr { u32x4 u; bf16x8 v; };
  for (int hx = blockIdx.y * kRopeHeads; hx < min(n_heads, (int)(blockIdx.y + 1) * kRopeHeads); ++hx) {
    // hx is the head of the input rows: a key/value head for keys, a query head for queries (which then
    // uses the rotation of key/value head hx / G and its own columns of q_lat)
    const int h = KEYS ? hx : hx / g.G, jq = KEYS ? 0 : hx % g.G;
    const int r = g.koff_r[h + 1] - g.koff_r[h];
    const uint16_t* X = static_cast<const uint16_t*>(g.A) + (int64_t)hx * g.d_head;  // row stride lda = heads * d_head
    const uint16_t* Rt = static_cast<const uint16_t*>(g.B) + (int64_t)g.koff_r[h] * g.d_head;
    // the rows of this head, rotated
    Fr af[2][4];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int col = 32 * ks + 8 * lg;
        u32x4 out = {0, 0, 0, 0};
        if (tok[t] >= 0 && col < g.d_head) {
          const u32x4 raw = *reinterpret_cast<const u32x4*>(X + (int64_t)tok[t] * g.lda + col);
          const float cc[4] = {cs[t][ks].x, cs[t][ks].y, cs[t][ks].z, cs[t][ks].w};
          const float ss[4] = {sn[t][ks].x, sn[t][ks].y, sn[t][ks].z, sn[t][ks].w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float xe = __uint_as_float(raw[j] << 16), xo = __uint_as_float(raw[j] & 0xffff0000u);
            out[j] = cvt_pk_bf16(xe * cc[j] - xo * ss[j], xe * ss[j] + xo * cc[j]);
          }
        }
        af[t][ks].u = out;
      }
    __syncthreads();   // every wave is done with the previous head's rotation rows
    {
      const int cpr = g.d_head / 8;
      for (int i = tid; i < r * cpr; i += 256) {
        const int row = i / cpr, c = i - row * cpr;
        *reinterpret_cast<u32x4*>(&lds_b[row * kRowsBRow + c * 8]) = *reinterpret_cast<const u32x4*>(Rt + (int64_t)row * g.d_head + c * 8);
      }
    }
    __syncthreads();
    for (int n0 = 0; n0 < r; n0 += 16) {
      f32x4 acc[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        if (ks >= ksteps) break;
        Fr bq;
        const int col = 32 * ks + 8 * lg;
        bq.u = col < g.d_head ? *reinterpret_cast<const u32x4*>(&lds_b[(n0 + ln) * kRowsBRow + col]) : u32x4{0, 0, 0, 0};
#pragma unroll
        for (int t = 0; t < 2; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bq.v, af[t][ks].v, acc[t], 0, 0, 0);
      }
      // register e of lane l: latent column n0 + 4 * (l / 16) + e of token row l % 16
      const int n = n0 + 4 * lg;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        if (tok[t] < 0) continue;
        if constexpr (KEYS) {
          const int64_t dst = tok_dst[t] + (int64_t)g.max_seq * g.koff_r[h] + (int64_t)g.tok_pos[tok[t]] * r + n;
          if (g.cache_fp4) {   // four consecutive columns: two bytes
            const uint32_t w = fp4_pair(acc[t][0], acc[t][1]) | (fp4_pair(acc[t][2], acc[t][3]) << 8);
            *reinterpret_cast<uint16_t*>(static_cast<uint8_t*>(g.C) + (dst >> 1)) = (uint16_t)w;
          } else if (g.cache_fp8) {
            auto sat = [](float v) { return fminf(fmaxf(v, -448.f), 448.f); };
            uint32_t w = __builtin_amdgcn_cvt_pk_fp8_f32(sat(acc[t][0]), sat(acc[t][1]), 0u, false);
            w = __builtin_amdgcn_cvt_pk_fp8_f32(sat(acc[t][2]), sat(acc[t][3]), w, true);
            *reinterpret_cast<uint32_t*>(static_cast<uint8_t*>(g.C) + dst) = w;
          } else {
            uint2 w;
            w.x = cvt_pk_bf16(acc[t][0], acc[t][1]);
            w.y = cvt_pk_bf16(acc[t][2], acc[t][3]);
            *reinterpret_cast<uint2*>(static_cast<uint16_t*>(g.C) + dst) = w;
          }
        } else {
          TC* dst = static_cast<TC*>(g.C) + (int64_t)tok[t] * g.G * g.RK + g.G * g.koff_r[h] + jq * r + n;
          if constexpr (sizeof(TC) == 4) {
            *reinterpret_cast<f32x4*>(dst) = acc[t];
          } else {
            uint2 w;
            w.x = cvt_pk_bf16(acc[t][0], acc[t][1]);
            w.y = cvt_pk_bf16(acc[t][2], acc[t][3]);
            *reinterpret_cast<uint2*>(dst) = w;
          }
        }
      }
    }
  }
}

static void fill_tables(GemmArgs& a, const fdc_layout* lay, int layer) {
  const int H = lay->H;
  a.H = H, a.d_head = lay->d_head, a.max_seq = lay->max_seq, a.max_batch = lay->max_batch;
  a.G = lay->G;
  a.RK = lay->RK(layer), a.RV = lay->RV(layer);
  std::copy_n(&lay->koff_r[(size_t)layer * (H + 1)], H + 1, a.koff_r);
  std::copy_n(&lay->voff_r[(size_t)layer * (H + 1)], H + 1, a.voff_r);
}

// Launches the kernel for the layout's dtype. a_f32 / c_f32 say how A and C are stored in a
// bf16 layout (activations coming from / going to fp32 tensors).
static fdc_status launch(const fdc_layout* lay, const GemmArgs& a, int groups, int n_max, bool a_f32, bool c_f32,
                         hipStream_t st) {
  if (a.M == 0 || n_max == 0) return FDC_OK;
  if (lay->dtype == FDC_F32) {
    const dim3 grid((n_max + 15) / 16, (a.M + 15) / 16, groups);
    hipLaunchKernelGGL(gemm_f32_kernel<float>, grid, dim3(256), 0, st, a);
  } else if (a.M <= 64 && a.mode == kAbsorbQuery && !a_f32 && a.K <= 128 && a.K % 8 == 0) {
    const dim3 grid((n_max + 15) / 16, groups);
    if (c_f32) hipLaunchKernelGGL(absorb_query_small_kernel<float>, grid, dim3(64), 0, st, a);
    else hipLaunchKernelGGL(absorb_query_small_kernel<uint16_t>, grid, dim3(64), 0, st, a);
  } else if ((a.mode == kAbsorbQuery || a.mode == kFold) && !a_f32 && a.K <= 128 && a.K % 8 == 0 && n_max <= 128 &&
             a.lda % 8 == 0 && a.ldb % 8 == 0 && a.ldc % 4 == 0 &&
             ((int64_t)a.M * a.lda + a.K) * 2 < ((int64_t)1 << 31)) {   // the kernel reads A through a 32-bit buffer range
    const dim3 grid((a.M + kRowsPerWg - 1) / kRowsPerWg, groups);
    if (c_f32) hipLaunchKernelGGL(grouped_rows_kernel<float>, grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL(grouped_rows_kernel<uint16_t>, grid, dim3(256), 0, st, a);
  } else if (a.M <= 16 && (a.mode == kPlain || a.mode == kProject)) {
    if (a_f32 && c_f32) launch_skinny16<float, float>(a, st);
    else if (a_f32) launch_skinny16<float, uint16_t>(a, st);
    else if (c_f32) launch_skinny16<uint16_t, float>(a, st);
    else launch_skinny16<uint16_t, uint16_t>(a, st);
  } else if (a.M <= 64 && (a.mode == kPlain || a.mode == kProject)) {
    if (a_f32 && c_f32) launch_skinny<float, float>(a, st);
    else if (a_f32) launch_skinny<float, uint16_t>(a, st);
    else if (c_f32) launch_skinny<uint16_t, float>(a, st);
    else launch_skinny<uint16_t, uint16_t>(a, st);
  } else if (!a_f32 && groups == 1 && (a.mode == kPlain || a.mode == kProject) && a.K % 8 == 0 && a.lda % 8 == 0 &&
             a.ldb % 8 == 0 && !(a.mode == kProject && a.cache_fp4)) {   // E2M1 caches take the per-element epilogue below
    GemmArgs b = a;
    b.nt = (a.N + DN - 1) / DN;
    const int tiles = b.nt * ((a.M + DM - 1) / DM);
    const int slots = (tiles + 7) / 8 * 8;
    int cus = 0;
    FDC_HIP_CHECK(device_compute_units(&cus));
    cus = std::max(cus, 8) / 8 * 8;
    const int full = slots / cus * cus, last = slots - full;   // slots of complete rounds, of the last round
    const bool cut = last > 0 && last <= cus / 2;
    b.split_from = cut ? full : INT_MAX;
    const dim3 grid(cut ? full + 2 * last : slots);
    if (c_f32) hipLaunchKernelGGL(gemm_dma_kernel<float>, grid, dim3(512), 0, st, b);
    else hipLaunchKernelGGL(gemm_dma_kernel<uint16_t>, grid, dim3(512), 0, st, b);
  } else {
    GemmArgs b = a;
    b.nt = (n_max + BN - 1) / BN;
    const int tiles = b.nt * ((a.M + BM - 1) / BM);
    const dim3 grid((tiles + 7) / 8 * 8, 1, groups);
    if (a_f32 && c_f32) hipLaunchKernelGGL((gemm_bf16_kernel<float, float>), grid, dim3(256), 0, st, b);
    else if (a_f32) hipLaunchKernelGGL((gemm_bf16_kernel<float, uint16_t>), grid, dim3(256), 0, st, b);
    else if (c_f32) hipLaunchKernelGGL((gemm_bf16_kernel<uint16_t, float>), grid, dim3(256), 0, st, b);
    else hipLaunchKernelGGL((gemm_bf16_kernel<uint16_t, uint16_t>), grid, dim3(256), 0, st, b);
  }
  FDC_HIP_CHECK(hipGetLastError());
  return FDC_OK;
}

static fdc_status check_common(const char* fn, const fdc_layout* lay, int layer, int T) {
  if (!lay) FDC_FAIL(FDC_INVALID_ARG, "%s: layout is NULL", fn);
  if (layer < 0 || layer >= lay->L) FDC_FAIL(FDC_BAD_SHAPE, "%s: layer %d outside [0, %d)", fn, layer, lay->L);
  if (T < 0) FDC_FAIL(FDC_BAD_SHAPE, "%s: T = %d is negative", fn, T);
  if (lay->H > kMaxHeads) FDC_FAIL(FDC_BAD_SHAPE, "%s: more than %d heads", fn, kMaxHeads);
  return FDC_OK;
}

}  // namespace fdc

using namespace fdc;

extern "C" {

fdc_status fdc_project_latent_kv(const fdc_layout* lay, int layer, const void* x, int T, const int32_t* tok_batch,
                                 const int32_t* tok_pos, const void* A_cat_t, void* k_cache, void* v_cache,
                                 int32_t* status, void* stream) {
  fdc_status s = check_common("fdc_project_latent_kv", lay, layer, T);
  if (s != FDC_OK) return s;
  if (T == 0) return FDC_OK;
  if (!x || !tok_batch || !tok_pos || !A_cat_t || !v_cache)
    FDC_FAIL(FDC_INVALID_ARG, "fdc_project_latent_kv: NULL argument");
  if (!aligned16(x) || !aligned16(A_cat_t) || (k_cache && !aligned16(k_cache)) || !aligned16(v_cache))
    FDC_FAIL(FDC_BAD_ALIGNMENT, "fdc_project_latent_kv: pointers must be 16-byte aligned");
  GemmArgs a{};
  fill_tables(a, lay, layer);
  a.A = x, a.B = A_cat_t, a.C = k_cache, a.C2 = v_cache;
  a.lda = lay->d_model, a.ldb = lay->d_model, a.ldc = 0;
  a.v_only = k_cache == nullptr;
  a.cache_fp8 = lay->dtype == FDC_FP8, a.cache_fp4 = lay->dtype == FDC_FP4;
  a.M = T, a.N = a.v_only ? a.RV : a.RK + a.RV, a.K = lay->d_model;
  a.mode = kProject;
  a.tok_batch = tok_batch, a.tok_pos = tok_pos, a.fault = status;
  return launch(lay, a, 1, a.N, false, false, static_cast<hipStream_t>(stream));
}

fdc_status fdc_absorb_query(const fdc_layout* lay, int layer, const void* q, int T, const void* Bk, void* q_lat,
                            fdc_dtype q_lat_dtype, void* stream) {
  fdc_status s = check_common("fdc_absorb_query", lay, layer, T);
  if (s != FDC_OK) return s;
  if (T == 0) return FDC_OK;
  if (!q || !Bk || !q_lat) FDC_FAIL(FDC_INVALID_ARG, "fdc_absorb_query: NULL argument");
  if (!aligned16(q) || !aligned16(Bk) || !aligned16(q_lat))
    FDC_FAIL(FDC_BAD_ALIGNMENT, "fdc_absorb_query: pointers must be 16-byte aligned");
  if (q_lat_dtype != FDC_BF16 && q_lat_dtype != FDC_F32) FDC_FAIL(FDC_UNSUPPORTED_DTYPE, "fdc_absorb_query: q_lat_dtype");
  if (lay->dtype == FDC_F32 && q_lat_dtype != FDC_F32)
    FDC_FAIL(FDC_UNSUPPORTED_DTYPE, "fdc_absorb_query: an fp32 layout writes fp32 q_lat");
  GemmArgs a{};
  fill_tables(a, lay, layer);
  a.A = q, a.B = Bk, a.C = q_lat;
  a.lda = (int64_t)lay->H * lay->G * lay->d_head, a.ldb = lay->d_head, a.ldc = (int64_t)lay->G * a.RK;
  a.M = T, a.N = 0, a.K = lay->d_head;
  a.mode = kAbsorbQuery;
  int n_max = 0;
  for (int h = 0; h < lay->H; ++h) n_max = std::max(n_max, lay->rk[(size_t)layer * lay->H + h]);
  return launch(lay, a, lay->H * lay->G, n_max, false, q_lat_dtype == FDC_F32, static_cast<hipStream_t>(stream));
}

fdc_status fdc_project_and_absorb_query(const fdc_layout* lay, int layer, const void* x, int T,
                                        const int32_t* tok_batch, const int32_t* tok_pos, const void* A_cat_t,
                                        void* k_cache, void* v_cache, const void* q, const void* Bk, void* q_lat,
                                        fdc_dtype q_lat_dtype, int32_t* status, void* stream) {
  // one launch only where both halves take their few-row kernels; otherwise the two calls in turn
  if (!lay || lay->dtype == FDC_F32 || T < 1 || T > 16 || layer < 0 || layer >= lay->L || !x || !tok_batch ||
      !tok_pos || !A_cat_t || !v_cache || !q || !Bk || !q_lat || !aligned16(x) || !aligned16(A_cat_t) ||
      (k_cache && !aligned16(k_cache)) || !aligned16(v_cache) || !aligned16(q) || !aligned16(Bk) ||
      !aligned16(q_lat) || (q_lat_dtype != FDC_BF16 && q_lat_dtype != FDC_F32) || lay->H > kMaxHeads) {
    fdc_status s = fdc_project_latent_kv(lay, layer, x, T, tok_batch, tok_pos, A_cat_t, k_cache, v_cache, status, stream);
    if (s != FDC_OK) return s;
    return fdc_absorb_query(lay, layer, q, T, Bk, q_lat, q_lat_dtype, stream);
  }
  GemmArgs p{};
  fill_tables(p, lay, layer);
  p.A = x, p.B = A_cat_t, p.C = k_cache, p.C2 = v_cache;
  p.lda = lay->d_model, p.ldb = lay->d_model, p.ldc = 0;
  p.v_only = k_cache == nullptr;
  p.cache_fp8 = lay->dtype == FDC_FP8, p.cache_fp4 = lay->dtype == FDC_FP4;
  p.M = T, p.N = p.v_only ? p.RV : p.RK + p.RV, p.K = lay->d_model;
  p.mode = kProject;
  p.tok_batch = tok_batch, p.tok_pos = tok_pos, p.fault = status;
  GemmArgs a{};
  fill_tables(a, lay, layer);
  a.A = q, a.B = Bk, a.C = q_lat;
  a.lda = (int64_t)lay->H * lay->G * lay->d_head, a.ldb = lay->d_head, a.ldc = (int64_t)lay->G * a.RK;
  a.M = T, a.N = 0, a.K = lay->d_head;
  a.mode = kAbsorbQuery;
  int n_max = 0;
  for (int h = 0; h < lay->H; ++h) n_max = std::max(n_max, lay->rk[(size_t)layer * lay->H + h]);
  const int col_tiles = (n_max + 15) / 16, jobs = col_tiles * lay->H * lay->G;
  const int n_proj = (p.N + 15) / 16;
  hipStream_t st = static_cast<hipStream_t>(stream);
  auto go = [&](auto kern, int waves) {
    const size_t lds = (size_t)waves * 16 * kSkinnyRow * sizeof(uint16_t);
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds) != hipSuccess) return;
    hipLaunchKernelGGL(kern, dim3(n_proj + (jobs + waves - 1) / waves), dim3(waves * 64), lds, st, p, a, n_proj, col_tiles);
  };
  const bool f32 = q_lat_dtype == FDC_F32;
  if (p.K > 2048) {
    if (f32) go(decode_prologue_kernel<float, 8>, 8);
    else go(decode_prologue_kernel<uint16_t, 8>, 8);
  } else {
    if (f32) go(decode_prologue_kernel<float, 4>, 4);
    else go(decode_prologue_kernel<uint16_t, 4>, 4);
  }
  FDC_HIP_CHECK(hipGetLastError());
  return FDC_OK;
}

fdc_status fdc_absorb_output(const fdc_layout* lay, int layer, int mode, const void* Bv, const void* Wo_t, void* Mt,
                             const void* o_lat, fdc_dtype o_lat_dtype, int T, void* y, fdc_dtype y_dtype,
                             void* stream) {
  fdc_status s = check_common("fdc_absorb_output", lay, layer, T);
  if (s != FDC_OK) return s;
  if (!Mt || !aligned16(Mt)) FDC_FAIL(FDC_INVALID_ARG, "fdc_absorb_output: Mt is NULL or not 16-byte aligned");
  GemmArgs a{};
  fill_tables(a, lay, layer);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (mode == FDC_FOLD) {
    if (!Bv || !Wo_t) FDC_FAIL(FDC_INVALID_ARG, "fdc_absorb_output(FOLD): NULL argument");
    if (!aligned16(Bv) || !aligned16(Wo_t)) FDC_FAIL(FDC_BAD_ALIGNMENT, "fdc_absorb_output(FOLD): alignment");
    a.A = Wo_t, a.B = Bv, a.C = Mt;
    a.lda = (int64_t)lay->H * lay->G * lay->d_head, a.ldb = lay->d_head, a.ldc = (int64_t)lay->G * a.RV;
    a.M = lay->d_model, a.N = 0, a.K = lay->d_head;
    a.mode = kFold;
    int n_max = 0;
    for (int h = 0; h < lay->H; ++h) n_max = std::max(n_max, lay->rv[(size_t)layer * lay->H + h]);
    return launch(lay, a, lay->H * lay->G, n_max, false, lay->dtype == FDC_F32, st);
  }
  if (mode == FDC_APPLY) {
    if (T == 0) return FDC_OK;
    if (!o_lat || !y) FDC_FAIL(FDC_INVALID_ARG, "fdc_absorb_output(APPLY): NULL argument");
    if (!aligned16(o_lat) || !aligned16(y)) FDC_FAIL(FDC_BAD_ALIGNMENT, "fdc_absorb_output(APPLY): alignment");
    for (fdc_dtype d : {o_lat_dtype, y_dtype})
      if (d != FDC_BF16 && d != FDC_F32) FDC_FAIL(FDC_UNSUPPORTED_DTYPE, "fdc_absorb_output(APPLY): dtype");
    if (lay->dtype == FDC_F32 && (o_lat_dtype != FDC_F32 || y_dtype != FDC_F32))
      FDC_FAIL(FDC_UNSUPPORTED_DTYPE, "fdc_absorb_output(APPLY): an fp32 layout takes and writes fp32");
    a.A = o_lat, a.B = Mt, a.C = y;
    a.lda = (int64_t)lay->G * a.RV, a.ldb = (int64_t)lay->G * a.RV, a.ldc = lay->d_model;
    a.M = T, a.N = lay->d_model, a.K = lay->G * a.RV;
    a.mode = kPlain;
    return launch(lay, a, 1, a.N, o_lat_dtype == FDC_F32, y_dtype == FDC_F32, st);
  }
  FDC_FAIL(FDC_INVALID_ARG, "fdc_absorb_output: mode %d", mode);
}

static fdc_status rope_common(const char* fn, const fdc_layout* lay, int layer, const void* x, int T,
                              const int32_t* tok_pos, const float* cos_t, const float* sin_t, int n_pos,
                              const void* R_t, void* out, GemmArgs* a) {
  fdc_status s = check_common(fn, lay, layer, T);
  if (s != FDC_OK) return s;
  if (lay->dtype == FDC_F32) FDC_FAIL(FDC_UNSUPPORTED_DTYPE, "%s: bf16 and E4M3 layouts only", fn);
  if (!x || !tok_pos || !cos_t || !sin_t || !R_t || !out) FDC_FAIL(FDC_INVALID_ARG, "%s: NULL argument", fn);
  if (n_pos <= 0) FDC_FAIL(FDC_BAD_SHAPE, "%s: n_pos must be positive", fn);
  if (!aligned16(x) || !aligned16(cos_t) || !aligned16(sin_t) || !aligned16(R_t) || !aligned16(out))
    FDC_FAIL(FDC_BAD_ALIGNMENT, "%s: pointers must be 16-byte aligned", fn);
  fill_tables(*a, lay, layer);
  a->A = x, a->B = R_t, a->C = out;
  a->lda = (int64_t)lay->H * lay->d_head;   // key rows; the query entry point widens it to the query heads
  a->M = T, a->K = lay->d_head;
  a->tok_pos = tok_pos, a->rope_cos = cos_t, a->rope_sin = sin_t, a->n_pos = n_pos;
  return FDC_OK;
}

fdc_status fdc_rope_absorb_query(const fdc_layout* lay, int layer, const void* q, int T, const int32_t* tok_pos,
                                 const float* cos_t, const float* sin_t, int n_pos, const void* R_t, void* q_lat,
                                 fdc_dtype q_lat_dtype, int32_t* status, void* stream) {
  if (T == 0 && lay) return FDC_OK;
  GemmArgs a{};
  a.fault = status;
  fdc_status s = rope_common("fdc_rope_absorb_query", lay, layer, q, T, tok_pos, cos_t, sin_t, n_pos, R_t, q_lat, &a);
  if (s != FDC_OK) return s;
  if (q_lat_dtype != FDC_BF16 && q_lat_dtype != FDC_F32) FDC_FAIL(FDC_UNSUPPORTED_DTYPE, "fdc_rope_absorb_query: q_lat_dtype");
  a.lda = (int64_t)lay->H * lay->G * lay->d_head;
  const dim3 grid((T + kRopeRows - 1) / kRopeRows, (lay->H * lay->G + kRopeHeads - 1) / kRopeHeads);
  if (q_lat_dtype == FDC_F32)
    hipLaunchKernelGGL((rope_compress_kernel<float, false>), grid, dim3(256), 0, static_cast<hipStream_t>(stream), a);
  else
    hipLaunchKernelGGL((rope_compress_kernel<uint16_t, false>), grid, dim3(256), 0, static_cast<hipStream_t>(stream), a);
  FDC_HIP_CHECK(hipGetLastError());
  return FDC_OK;
}

fdc_status fdc_rope_compress_keys(const fdc_layout* lay, int layer, const void* k, int T, const int32_t* tok_batch,
                                  const int32_t* tok_pos, const float* cos_t, const float* sin_t, int n_pos,
                                  const void* R_t, void* k_cache, int32_t* status, void* stream) {
  if (T == 0 && lay) return FDC_OK;
  GemmArgs a{};
  a.fault = status;
  fdc_status s = rope_common("fdc_rope_compress_keys", lay, layer, k, T, tok_pos, cos_t, sin_t, n_pos, R_t, k_cache, &a);
  if (s != FDC_OK) return s;
  if (!tok_batch) FDC_FAIL(FDC_INVALID_ARG, "fdc_rope_compress_keys: tok_batch is NULL");
  a.tok_batch = tok_batch;
  a.cache_fp8 = lay->dtype == FDC_FP8, a.cache_fp4 = lay->dtype == FDC_FP4;
  const dim3 grid((T + kRopeRows - 1) / kRopeRows, (lay->H + kRopeHeads - 1) / kRopeHeads);
  hipLaunchKernelGGL((rope_compress_kernel<uint16_t, true>), grid, dim3(256), 0, static_cast<hipStream_t>(stream), a);
  FDC_HIP_CHECK(hipGetLastError());
  return FDC_OK;
}

}  // extern "C"
