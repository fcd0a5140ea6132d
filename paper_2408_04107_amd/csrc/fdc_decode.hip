// Decode attention on the latent KV cache (Section 5, step 7 of the paper: compressed Q', K', V'
// go into attention without decompression; Section 5.3: per-head tasks of uneven cost are balanced
// over the compute units).
//
// Design for gfx950. The work is one dot product and one axpy per cached element (1 flop per
// byte), so the kernel is a pure HBM stream. A worker is one wavefront. It walks the tiles the
// planner gave it; a tile is a token range of one (sequence, head) unit and therefore ONE
// contiguous span of K' and one of V'. Each lane issues 16-byte loads that are contiguous across
// the wave (1 KiB per load instruction). A row of rank r occupies L = r*sizeof(T)/16 lanes, padded
// to a power of two, so a dot product is finished with log2(L) DPP adds. Scores of a block of
// tokens go through a per-wave LDS strip, which (a) lets each score be exponentiated once instead
// of once per lane of its row and (b) decouples the lane mapping of K' rows (rank rk) from that
// of V' rows (rank rv). The softmax reference m is only raised when a block exceeds it by a
// margin, so most blocks need no cross-lane maximum and no rescale. Split units leave
// (m, l, acc) in a slot of their own (no atomics, deterministic) and a second small kernel merges
// them.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <mutex>

#include "fdc_internal.h"

namespace fdc {

// Wave-wide 16-byte loads of the wider operand per block: 8 KiB per wave in flight and side (4 to 16
// measured within 2 % of each other).
constexpr int kDecodeLoads = 8;
// The code caches take half as many: sixteen elements per load keep twice the widened values live, and with
// eight loads the E4M3 instance needs 152 registers (three wavefronts per SIMD, 76 us for layer 0 of the
// adaptive-rank config); with four it fits four wavefronts (112 registers, 69 us). 2 and 6 are slower again.
constexpr int kDecodeLoadsCodes = 4;
constexpr int kTokLanes = 64 * kDecodeLoads;
constexpr int kWavesPerBlock = kWorkersPerGroup;
constexpr int kLdsFloatsPerWave = kTokLanes > 256 ? kTokLanes : 256;  // a block of one-lane rows (E4M3, rank 16) has kTokLanes tokens

// Tokens per block: kDecodeLoads loads of the wider operand, at least one load of the narrower.
constexpr int block_tokens(int lk, int lv, int loads = kDecodeLoads) {
  int t = 64 * loads / (lk > lv ? lk : lv);
  const int need = 64 / (lk < lv ? lk : lv);
  return t > need ? t : need;
}
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kRaiseMargin = 6.0f;  // in log2 units: p never exceeds 2^6 between raises
constexpr int kBufferFlags = 0x00020000;  // word 3 of a gfx9 raw buffer descriptor: 32-bit data format

// Cache policy of the K'/V' stream: the "nt" (non-temporal) bit. Every cached byte is read exactly
// once per step, so it should not displace anything in L2 / the last-level cache; measured on
// MI355X a read-only stream reaches about 6.1 TB/s with default loads and about 7.0 TB/s with nt.
constexpr int kStreamPolicy = 2;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// ---- small device helpers -------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// Sum over aligned groups of L lanes (L a power of two); every lane of the group gets the sum.
template <int L>
__device__ __forceinline__ float group_sum(float v) {
  if constexpr (L >= 2) v += dpp<0xB1>(v);    // quad_perm [1,0,3,2]
  if constexpr (L >= 4) v += dpp<0x4E>(v);    // quad_perm [2,3,0,1]
  if constexpr (L >= 8) v += dpp<0x141>(v);   // row_half_mirror
  if constexpr (L >= 16) v += dpp<0x140>(v);  // row_mirror
  if constexpr (L >= 32) v += __shfl_xor(v, 16);
  if constexpr (L >= 64) v += __shfl_xor(v, 32);
  return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}

__device__ __forceinline__ void wave_lds_sync() {
  // LDS operations of one wavefront execute in order; this only stops the compiler from moving
  // LDS accesses of different lanes' data across the point.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <typename T>
struct Elem;
// EL elements per lane and load, BITS per element, Reg the loaded registers (a 16-byte load, 8 bytes for E2M1 so
// that the narrowest row, sixteen codes, is still one lane's load).
template <>
struct Elem<uint16_t> {  // bf16 bits
  static constexpr int EL = 8, BITS = 16, LOADS = kDecodeLoads;
  typedef u32x4 Reg;
  __device__ static __forceinline__ Reg load(__amdgpu_buffer_rsrc_t rsrc, int off) {
    return __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, kStreamPolicy);
  }
  __device__ static __forceinline__ void widen(const u32x4& r, float* f) {
    f[0] = __uint_as_float(r[0] << 16), f[1] = __uint_as_float(r[0] & 0xffff0000u);
    f[2] = __uint_as_float(r[1] << 16), f[3] = __uint_as_float(r[1] & 0xffff0000u);
    f[4] = __uint_as_float(r[2] << 16), f[5] = __uint_as_float(r[2] & 0xffff0000u);
    f[6] = __uint_as_float(r[3] << 16), f[7] = __uint_as_float(r[3] & 0xffff0000u);
  }
};
template <>
struct Elem<uint8_t> {  // OCP E4M3 codes: sixteen elements per 16-byte load, decoded in pairs (v_cvt_pk_f32_fp8)
  static constexpr int EL = 16, BITS = 8, LOADS = kDecodeLoadsCodes;
  typedef u32x4 Reg;
  __device__ static __forceinline__ Reg load(__amdgpu_buffer_rsrc_t rsrc, int off) {
    return __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, kStreamPolicy);
  }
  __device__ static __forceinline__ void widen(const u32x4& r, float* f) {
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const auto lo = __builtin_amdgcn_cvt_pk_f32_fp8(r[w], false);  // bytes 0, 1 of the word
      const auto hi = __builtin_amdgcn_cvt_pk_f32_fp8(r[w], true);   // bytes 2, 3
      f[4 * w + 0] = lo[0], f[4 * w + 1] = lo[1], f[4 * w + 2] = hi[0], f[4 * w + 3] = hi[1];
    }
  }
};
template <>
struct Elem<fp4_t> {  // OCP E2M1 codes: sixteen elements per 8-byte load, decoded a byte (two codes) at a time
  static constexpr int EL = 16, BITS = 4, LOADS = kDecodeLoadsCodes;
  typedef u32x2 Reg;
  __device__ static __forceinline__ Reg load(__amdgpu_buffer_rsrc_t rsrc, int off) {
    return __builtin_amdgcn_raw_buffer_load_b64(rsrc, off, 0, kStreamPolicy);
  }
  __device__ static __forceinline__ void widen(const u32x2& r, float* f) {
#pragma unroll
    for (int w = 0; w < 2; ++w) {
      const auto b0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(r[w], 1.0f, 0);   // byte 0: elements 8 w, 8 w + 1
      const auto b1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(r[w], 1.0f, 1);
      const auto b2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(r[w], 1.0f, 2);
      const auto b3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(r[w], 1.0f, 3);
      f[8 * w + 0] = b0[0], f[8 * w + 1] = b0[1], f[8 * w + 2] = b1[0], f[8 * w + 3] = b1[1];
      f[8 * w + 4] = b2[0], f[8 * w + 5] = b2[1], f[8 * w + 6] = b3[0], f[8 * w + 7] = b3[1];
    }
  }
};
template <>
struct Elem<float> {
  static constexpr int EL = 4, BITS = 32, LOADS = kDecodeLoads;
  typedef u32x4 Reg;
  __device__ static __forceinline__ Reg load(__amdgpu_buffer_rsrc_t rsrc, int off) {
    return __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, kStreamPolicy);
  }
  __device__ static __forceinline__ void widen(const u32x4& r, float* f) {
    f[0] = __uint_as_float(r[0]), f[1] = __uint_as_float(r[1]);
    f[2] = __uint_as_float(r[2]), f[3] = __uint_as_float(r[3]);
  }
};

// ---- one tile -----------------------------------------------------------------------------
// LK / LV: lanes per K' / V' row (power of two >= rank * sizeof(T) / 16).
template <typename T, int LK, int LV>
__device__ __forceinline__ void decode_tile(const DecTile& td, const float* __restrict__ q_lat,
                                            const T* __restrict__ kc, const T* __restrict__ vc, float scale_log2,
                                            float* __restrict__ o_lat, float* __restrict__ partials, float* lds,
                                            const int lane) {
  constexpr int EL = Elem<T>::EL;
  constexpr int TB = block_tokens(LK, LV, Elem<T>::LOADS);              // tokens per block
  constexpr int RK_ROWS = 64 / LK, RV_ROWS = 64 / LV;                    // rows per wave-wide load
  constexpr int NK = TB / RK_ROWS, NV = TB / RV_ROWS;                    // loads per lane per block
  constexpr int NS = (TB + 63) / 64;                                     // scores per lane per block
  static_assert(NK >= 1 && NV >= 1 && TB <= kLdsFloatsPerWave, "block shape");

  const int rk = td.rk_rv & 0xffff, rv = td.rk_rv >> 16;
  const int len = td.len;
  const int ck = lane % LK, sk = lane / LK;
  const int cv = lane % LV, sv = lane / LV;
  const bool k_on = ck * EL < rk, v_on = cv * EL < rv;

  // q' of the lane's column group, pre-multiplied by scale * log2(e); padded lanes hold zeros
  float qf[EL];
  {
    const float* qp = q_lat + td.q_elem + (k_on ? ck * EL : 0);
    const float qs = k_on ? scale_log2 : 0.f;
#pragma unroll
    for (int j = 0; j < EL; ++j) qf[j] = qp[j] * qs;
  }

  // The tile's K' and V' spans as raw buffers: loads past the span (rows >= len in the last
  // block) and loads of padded lanes (offset forced out of range) return zeros in hardware, so
  // the stream has no branches. The range check covers the VGPR offset only, so the whole
  // row offset is kept there.
  constexpr int BITS = Elem<T>::BITS, LB = EL * BITS / 8;   // bits per element, bytes per lane and load
  const int k_row_bytes = rk * BITS / 8, v_row_bytes = rv * BITS / 8;
  const __amdgpu_buffer_rsrc_t k_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(reinterpret_cast<const uint8_t*>(kc) + td.k_elem * BITS / 8), 0, len * k_row_bytes, kBufferFlags);
  const __amdgpu_buffer_rsrc_t v_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(reinterpret_cast<const uint8_t*>(vc) + td.v_elem * BITS / 8), 0, len * v_row_bytes, kBufferFlags);
  const uint32_t k_lane = k_on ? (uint32_t)(sk * k_row_bytes + ck * LB) : 0x80000000u;
  const uint32_t v_lane = v_on ? (uint32_t)(sv * v_row_bytes + cv * LB) : 0x80000000u;

  typename Elem<T>::Reg kreg[NK], vreg[NV];
  auto load_k = [&](int t0) {
    const uint32_t base = k_lane + (uint32_t)(t0 * k_row_bytes);
#pragma unroll
    for (int i = 0; i < NK; ++i)
      kreg[i] = Elem<T>::load(k_rsrc, (int)(base + (uint32_t)(i * RK_ROWS * k_row_bytes)));
  };
  auto load_v = [&](int t0) {
    const uint32_t base = v_lane + (uint32_t)(t0 * v_row_bytes);
#pragma unroll
    for (int i = 0; i < NV; ++i)
      vreg[i] = Elem<T>::load(v_rsrc, (int)(base + (uint32_t)(i * RV_ROWS * v_row_bytes)));
  };

  float acc[EL];
#pragma unroll
  for (int j = 0; j < EL; ++j) acc[j] = 0.f;
  float m = -INFINITY, l = 0.f;

  load_k(0);
  __builtin_amdgcn_sched_barrier(0);  // keep issue order K' then V': the wait counters rely on it
  load_v(0);
  __builtin_amdgcn_sched_barrier(0);
  for (int t0 = 0; t0 < len; t0 += TB) {
    // scores of the block -> LDS strip
#pragma unroll
    for (int i = 0; i < NK; ++i) {
      float f[EL];
      Elem<T>::widen(kreg[i], f);
      float d = 0.f;
#pragma unroll
      for (int j = 0; j < EL; ++j) d = fmaf(qf[j], f[j], d);
      d = group_sum<LK>(d);
      const int r = i * RK_ROWS + sk;
      if (t0 + r >= len) d = -INFINITY;
      lds[r] = d;  // every lane of the row's group holds the sum; same-address writes need no branch
    }
    __builtin_amdgcn_sched_barrier(0);
    load_k(t0 + TB);  // past the end of the tile the hardware range check returns zeros
    __builtin_amdgcn_sched_barrier(0);
    wave_lds_sync();

    // one exponential per score; raise the reference only when a block beats it by the margin
    float s[NS], loc = -INFINITY;
#pragma unroll
    for (int j = 0; j < NS; ++j) {
      const int idx = lane + 64 * j;
      s[j] = idx < TB ? lds[idx] : -INFINITY;
      loc = fmaxf(loc, s[j]);
    }
    if (__any(loc > m + kRaiseMargin)) {
      const float nm = fmaxf(m, wave_max(loc));
      const float alpha = __builtin_amdgcn_exp2f(m - nm);  // m = -inf on the first block: 0
      l *= alpha;
#pragma unroll
      for (int j = 0; j < EL; ++j) acc[j] *= alpha;
      m = nm;
    }
#pragma unroll
    for (int j = 0; j < NS; ++j) {
      const int idx = lane + 64 * j;
      const float p = __builtin_amdgcn_exp2f(s[j] - m);
      l += p;
      if (idx < TB) lds[idx] = p;
    }
    wave_lds_sync();

    // acc += p * V'
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const float p = lds[i * RV_ROWS + sv];
      float f[EL];
      Elem<T>::widen(vreg[i], f);
#pragma unroll
      for (int j = 0; j < EL; ++j) acc[j] = fmaf(p, f[j], acc[j]);
    }
    __builtin_amdgcn_sched_barrier(0);
    load_v(t0 + TB);
    __builtin_amdgcn_sched_barrier(0);
    wave_lds_sync();
  }

  // tile result: l over all lanes, acc over the lanes that share a column group
  l = group_sum<64>(l);
#pragma unroll
  for (int o = LV; o < 64; o <<= 1) {
#pragma unroll
    for (int j = 0; j < EL; ++j) acc[j] += __shfl_xor(acc[j], o);
  }
  if (sv == 0 && v_on) {
    if (td.slot < 0) {
      const float inv = 1.f / l;
      float* o = o_lat + td.o_elem + cv * EL;
#pragma unroll
      for (int j = 0; j < EL; ++j) o[j] = acc[j] * inv;
    } else {
      float* pp = partials + (int64_t)td.slot * kPartialStride;
#pragma unroll
      for (int j = 0; j < EL; ++j) pp[4 + cv * EL + j] = acc[j];
      if (cv == 0) pp[0] = m, pp[1] = l;
    }
  }
}

// log2 of the padded lanes-per-row: rank r needs r * sizeof(T) / 16 lanes.
template <typename T>
__device__ __forceinline__ int lane_class(int r) {
  const int lanes = r / Elem<T>::EL;  // 1..8 (E4M3), 2..16 (bf16), 4..32 (f32)
  return lanes <= 1 ? 0 : 32 - __builtin_clz(lanes - 1);  // ceil(log2(lanes))
}

template <typename T>
__global__ __launch_bounds__(kWavesPerBlock * 64) void decode_tiles_kernel(
    const DecWorker* __restrict__ workers, const DecTile* __restrict__ wtiles, const float* __restrict__ q_lat,
    const T* __restrict__ kc, const T* __restrict__ vc, float scale_log2, float* __restrict__ o_lat,
    float* __restrict__ partials, int n_workers, const int32_t* __restrict__ planned_len,
    const int32_t* __restrict__ seq_len, const int group_j) {
  __shared__ float lds_all[kWavesPerBlock][kLdsFloatsPerWave];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
  const int lane = threadIdx.x % 64;
  const int worker = blockIdx.x * kWavesPerBlock + wave;
  if (worker >= n_workers) return;
  float* lds = lds_all[wave];
  const DecWorker* hd = workers + worker;
  const int count = hd->count, begin = hd->begin;
  if (count == 0) return;
  DecTile td = hd->first;
  constexpr int BASE = Elem<T>::EL == 16 ? 0 : (Elem<T>::EL == 8 ? 1 : 2);  // smallest lane class (log2 lanes per row) of this element type
  for (int i = 0;;) {
    // the record of the next tile is requested before this one is streamed, so that a tile boundary does not
    // wait for it (the last iteration re-reads the current record: always a valid address)
    const DecTile next = wtiles[begin + min(i + 1, count - 1)];
    td.len = dec_tile_len(td, planned_len, seq_len);
    // query head group_j of the tile's group (0 for multi-head plans): its q', its o', its partial slot
    td.q_elem += group_j * (td.rk_rv & 0xffff), td.o_elem += group_j * (td.rk_rv >> 16);
    if (td.slot >= 0) td.slot += group_j * td.slot_stride;
    const int ck = lane_class<T>(td.rk_rv & 0xffff) - BASE, cvv = lane_class<T>(td.rk_rv >> 16) - BASE;
#define FDC_CASE(a, b)                                                                                      \
  case (a)*4 + (b):                                                                                         \
    decode_tile<T, (1 << ((a) + BASE)), (1 << ((b) + BASE))>(td, q_lat, kc, vc, scale_log2, o_lat, partials, lds, \
                                                             lane);                                                \
    break;
    switch (ck * 4 + cvv) {
      FDC_CASE(0, 0) FDC_CASE(0, 1) FDC_CASE(0, 2) FDC_CASE(0, 3)
      FDC_CASE(1, 0) FDC_CASE(1, 1) FDC_CASE(1, 2) FDC_CASE(1, 3)
      FDC_CASE(2, 0) FDC_CASE(2, 1) FDC_CASE(2, 2) FDC_CASE(2, 3)
      FDC_CASE(3, 0) FDC_CASE(3, 1) FDC_CASE(3, 2) FDC_CASE(3, 3)
      default: break;
    }
#undef FDC_CASE
    if (++i >= count) break;
    td = next;
  }
}

// ---- split-K merge --------------------------------------------------------------------------
// o' = sum_j acc_j 2^(m_j - M) / sum_j l_j 2^(m_j - M), M = max_j m_j, over the tiles j of a unit.
//
// Units cut into many tiles (long contexts): one workgroup of sixteen wavefronts per unit. Wave w
// takes the tiles w, w + 16, w + 32, ... eight at a time (every load of a batch in flight together;
// a lane owns two output columns) and keeps a running (M, L, acc) in registers; the sixteen wave
// states are then combined through LDS in wave order. A unit of 270 tiles costs three dependent
// rounds of loads per wave, where one thread per (column quad, tile group) walking its tiles one
// after the other took nine.
constexpr int kWideWaves = 16;
constexpr int kWideBatch = 8;
constexpr int kMergeWaveMax = 64;   // units of up to this many tiles belong to the one-wavefront kernel below

__global__ __launch_bounds__(kWideWaves * 64) void decode_merge_wide_kernel(const DecUnit* __restrict__ units,
                                                                            const float* __restrict__ partials,
                                                                            float* __restrict__ o_lat) {
  const DecUnit u = units[blockIdx.x];
  const int n = u.tile_end - u.tile_begin;
  const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
  if (n <= kMergeWaveMax) return;  // merged by decode_merge_wave_kernel (or, a single tile, final already)
  __shared__ float accs[kWideWaves][130];  // [w][0..127] acc, [128] L, [129] M
  const bool on = 2 * lane < u.rv;
  const float* base = partials + (int64_t)u.tile_begin * kPartialStride;
  float M = -INFINITY, L = 0.f, ax = 0.f, ay = 0.f;
  for (int j0 = wave; j0 < n; j0 += kWideWaves * kWideBatch) {
    float2 ml[kWideBatch], v[kWideBatch];
#pragma unroll
    for (int t = 0; t < kWideBatch; ++t) {
      const float* pp = base + (int64_t)min(j0 + kWideWaves * t, n - 1) * kPartialStride;  // past the end: a valid slot, weight 0
      ml[t] = *reinterpret_cast<const float2*>(pp);
      v[t] = *reinterpret_cast<const float2*>(pp + 4 + (on ? 2 * lane : 0));
    }
    float bm = M;
#pragma unroll
    for (int t = 0; t < kWideBatch; ++t) {
      if (j0 + kWideWaves * t >= n) ml[t].x = -INFINITY;
      bm = fmaxf(bm, ml[t].x);
    }
    const float w0 = __builtin_amdgcn_exp2f(M - bm);  // first batch: 2^(-inf) = 0
    L *= w0, ax *= w0, ay *= w0;
#pragma unroll
    for (int t = 0; t < kWideBatch; ++t) {
      const float w = __builtin_amdgcn_exp2f(ml[t].x - bm);
      L = fmaf(ml[t].y, w, L), ax = fmaf(v[t].x, w, ax), ay = fmaf(v[t].y, w, ay);
    }
    M = bm;
  }
  // a wave without tiles (n < 16) leaves M = -inf, L = 0: weight 0 below
  accs[wave][2 * lane] = ax, accs[wave][2 * lane + 1] = ay;
  if (lane == 0) accs[wave][128] = L, accs[wave][129] = M;
  __syncthreads();
  if (tid < u.rv) {
    float Mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < kWideWaves; ++k) Mx = fmaxf(Mx, accs[k][129]);
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int k = 0; k < kWideWaves; ++k) {
      const float w = __builtin_amdgcn_exp2f(accs[k][129] - Mx);
      num = fmaf(accs[k][tid], w, num), den = fmaf(accs[k][128], w, den);
    }
    o_lat[u.o_elem + tid] = num / den;
  }
}

// The same merge for units cut into a few tiles (every decode step at ordinary context lengths):
// one wavefront per unit, a lane owns two output columns, and the states are read sixteen at a time
// (all loads of a batch in flight together), so a unit costs two dependent memory round trips (its
// record, then its states) instead of three. States are combined in slot order.
constexpr int kMergeBatch = 16;
constexpr int kMergeWaves = 4;

__global__ __launch_bounds__(kMergeWaves * 64) void decode_merge_wave_kernel(const DecUnit* __restrict__ units,
                                                                             const float* __restrict__ partials,
                                                                             float* __restrict__ o_lat, int n_units) {
  const int unit = blockIdx.x * kMergeWaves + (int)(threadIdx.x / 64);
  if (unit >= n_units) return;
  const int lane = threadIdx.x % 64;
  const DecUnit u = units[unit];
  const int n = u.tile_end - u.tile_begin;
  if (n == 1 || n > kMergeWaveMax) return;  // one tile: the tile kernel wrote the normalised output itself; many: the wide kernel
  const bool on = 2 * lane < u.rv;
  if (n == 0) {
    if (on) *reinterpret_cast<float2*>(o_lat + u.o_elem + 2 * lane) = make_float2(0.f, 0.f);
    return;
  }
  const float* base = partials + (int64_t)u.tile_begin * kPartialStride;
  float M = -INFINITY, L = 0.f, ax = 0.f, ay = 0.f;
  for (int j0 = 0; j0 < n; j0 += kMergeBatch) {
    float2 ml[kMergeBatch], v[kMergeBatch];
#pragma unroll
    for (int t = 0; t < kMergeBatch; ++t) {
      const float* pp = base + (int64_t)min(j0 + t, n - 1) * kPartialStride;  // past the end: a valid slot, weight 0
      ml[t] = *reinterpret_cast<const float2*>(pp);
      v[t] = *reinterpret_cast<const float2*>(pp + 4 + (on ? 2 * lane : 0));
    }
    float bm = M;
#pragma unroll
    for (int t = 0; t < kMergeBatch; ++t) {
      if (j0 + t >= n) ml[t].x = -INFINITY;
      bm = fmaxf(bm, ml[t].x);
    }
    const float w0 = __builtin_amdgcn_exp2f(M - bm);  // first batch: 2^(-inf) = 0
    L *= w0, ax *= w0, ay *= w0;
#pragma unroll
    for (int t = 0; t < kMergeBatch; ++t) {
      const float w = __builtin_amdgcn_exp2f(ml[t].x - bm);
      L = fmaf(ml[t].y, w, L), ax = fmaf(v[t].x, w, ax), ay = fmaf(v[t].y, w, ay);
    }
    M = bm;
  }
  if (on) {
    const float inv = 1.f / L;
    *reinterpret_cast<float2*>(o_lat + u.o_elem + 2 * lane) = make_float2(ax * inv, ay * inv);
  }
}

}  // namespace fdc

using namespace fdc;

static thread_local hipEvent_t g_prof_start = nullptr, g_prof_stop = nullptr;

// Workspace of fdc_latent_attn_decode_static: plan tables and split-K partial states in device memory
// that belongs to the code object, so that the call allocates nothing. Every GPU the library runs on
// holds its own copy at its own address until the process ends. In host code the array's name is
// only a handle for hipGetSymbolAddress: the address kernels and copies use is the one that call
// returns, looked up once per device and kept below.
constexpr size_t kStaticScratchBytes = FDC_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
struct ScratchOfDevice {
  void* ptr = nullptr;           // device address of `scratch` on this GPU
  uint64_t resident_plan = 0;    // serial of the plan whose tables the array holds (0: none)
};
std::mutex g_scratch_mutex;
ScratchOfDevice g_scratch_of[kMaxDevices];
}  // namespace

extern "C" {

fdc_status fdc_profile_decode_events(void* start_event, void* stop_event) {
  if ((start_event == nullptr) != (stop_event == nullptr))
    FDC_FAIL(FDC_INVALID_ARG, "fdc_profile_decode_events: pass two events or two NULLs");
  g_prof_start = static_cast<hipEvent_t>(start_event);
  g_prof_stop = static_cast<hipEvent_t>(stop_event);
  return FDC_OK;
}

fdc_status fdc_suggest_workers(int kind, int32_t* n_workers) {
  if (!n_workers) FDC_FAIL(FDC_INVALID_ARG, "fdc_suggest_workers: NULL argument");
  int dev = 0;
  FDC_HIP_CHECK(hipGetDevice(&dev));
  hipDeviceProp_t prop;
  FDC_HIP_CHECK(hipGetDeviceProperties(&prop, dev));
  if (kind == 0) {
    int nb = 0;
    FDC_HIP_CHECK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, decode_tiles_kernel<uint16_t>,
                                                               kWavesPerBlock * 64, 0));
    *n_workers = prop.multiProcessorCount * std::max(nb, 1) * kWavesPerBlock;
  } else if (kind == 3) {
    int nb = 0;
    FDC_HIP_CHECK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, decode_tiles_kernel<uint8_t>,
                                                               kWavesPerBlock * 64, 0));
    *n_workers = prop.multiProcessorCount * std::max(nb, 1) * kWavesPerBlock;
  } else if (kind == 4) {
    int nb = 0;
    FDC_HIP_CHECK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, decode_tiles_kernel<fp4_t>,
                                                               kWavesPerBlock * 64, 0));
    *n_workers = prop.multiProcessorCount * std::max(nb, 1) * kWavesPerBlock;
  } else if (kind == 2) {
    int waves = 0;
    fdc_status st = decode_gqa_workers_per_cu(&waves);
    if (st != FDC_OK) return st;
    *n_workers = prop.multiProcessorCount * waves;
  } else if (kind == 1) {
    int nb = 0;
    fdc_status st = prefill_blocks_per_cu(&nb);
    if (st != FDC_OK) return st;
    *n_workers = prop.multiProcessorCount * std::max(nb, 1);
  } else {
    FDC_FAIL(FDC_INVALID_ARG, "fdc_suggest_workers: kind %d", kind);
  }
  return FDC_OK;
}

fdc_status fdc_plan_upload(const fdc_plan* plan, void* workspace, size_t workspace_bytes, void* stream) {
  if (!plan || !workspace) FDC_FAIL(FDC_INVALID_ARG, "fdc_plan_upload: NULL argument");
  if (workspace_bytes < plan->workspace_bytes)
    FDC_FAIL(FDC_WORKSPACE_TOO_SMALL, "fdc_plan_upload: workspace has %zu bytes, the plan needs %zu", workspace_bytes,
             plan->workspace_bytes);
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
    FDC_FAIL(FDC_BAD_ALIGNMENT, "fdc_plan_upload: workspace must be 256-byte aligned");
  FDC_HIP_CHECK(hipMemcpyAsync(workspace, plan->image.data(), plan->image.size(), hipMemcpyHostToDevice,
                               static_cast<hipStream_t>(stream)));
  return FDC_OK;
}

}  // extern "C"

static fdc_status decode_impl(const fdc_layout* lay, const fdc_plan* plan, const int32_t* lens, const void* q_lat,
                              const void* k_cache, const void* v_cache, float scale, void* o_lat, void* workspace,
                              size_t workspace_bytes, void* stream) {
  // a pending profiling request belongs to THIS call, whether it succeeds or not
  hipEvent_t ev0 = g_prof_start, ev1 = g_prof_stop;
  g_prof_start = g_prof_stop = nullptr;
  if (!lay || !plan || !q_lat || !k_cache || !v_cache || !o_lat || !workspace)
    FDC_FAIL(FDC_INVALID_ARG, "fdc_latent_attn_decode: NULL argument");
  if (plan->kind != 0 || plan->lay != lay) FDC_FAIL(FDC_INVALID_ARG, "fdc_latent_attn_decode: not a decode plan of this layout");
  if (!(scale > 0.f) || !(scale < 1e30f))
    FDC_FAIL(FDC_INVALID_ARG, "fdc_latent_attn_decode: scale must be positive and finite (the running softmax orders scores by scale * s)");
  if (workspace_bytes < plan->workspace_bytes)
    FDC_FAIL(FDC_WORKSPACE_TOO_SMALL, "fdc_latent_attn_decode: workspace has %zu bytes, the plan needs %zu",
             workspace_bytes, plan->workspace_bytes);
  if (!aligned16(q_lat) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(o_lat) ||
      (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
    FDC_FAIL(FDC_BAD_ALIGNMENT, "fdc_latent_attn_decode: pointers must be 16-byte aligned (workspace 256)");
  hipStream_t st = static_cast<hipStream_t>(stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  const DecTile* wtiles = reinterpret_cast<const DecTile*>(ws + plan->off_items);
  const DecUnit* units = reinterpret_cast<const DecUnit*>(ws + plan->off_units);
  const DecWorker* heads = reinterpret_cast<const DecWorker*>(ws + plan->off_worker_ptr);
  float* partials = reinterpret_cast<float*>(ws + plan->off_partials);
  const int32_t* planned = reinterpret_cast<const int32_t*>(ws + plan->off_lens);
  const int W = plan->n_workers;
  const dim3 grid((W + kWavesPerBlock - 1) / kWavesPerBlock), block(kWavesPerBlock * 64);
  const float scale_log2 = scale * kLog2e;
  // Grouped queries over a bf16 or E4M3 cache stream a tile once for the whole group (matrix-core kernel).
  // The other element types have no such kernel: the multi-head kernel runs once per query head of the
  // group, each pass over the same tiles with that head's q', o' and partial slots (g times the traffic).
  const bool per_head_passes = plan->G > 1 && (lay->dtype == FDC_F32 || lay->dtype == FDC_FP4);
  const int n_pass = per_head_passes ? plan->G : 1;
  if (plan->on_device || !plan->item_b.empty()) {   // a device plan's tile count is not known here: empty workers return at once
    // a profiling request attaches its two events to the tile kernel's own dispatch (its begin and its end)
    // (with several passes: the start event on the first pass, the stop event on the last)
#define FDC_LAUNCH_TILES(kern, ...)                                                                              \
  do {                                                                                                           \
    for (int j = 0; j < n_pass; ++j) {                                                                           \
      hipEvent_t e0 = j == 0 ? ev0 : nullptr, e1 = j == n_pass - 1 ? ev1 : nullptr;                              \
      if (e0 || e1) hipExtLaunchKernelGGL(kern, grid, block, 0, st, e0, e1, 0, __VA_ARGS__, j);                  \
      else hipLaunchKernelGGL(kern, grid, block, 0, st, __VA_ARGS__, j);                                         \
    }                                                                                                            \
  } while (0)
    if (plan->G > 1 && !per_head_passes) {
      fdc_status gs = launch_decode_gqa(heads, wtiles, static_cast<const float*>(q_lat), k_cache, v_cache,
                                        lay->dtype == FDC_FP8, scale, static_cast<float*>(o_lat), partials, W, planned, lens,
                                        ev0, ev1, st);
      if (gs != FDC_OK) return gs;
    } else if (lay->dtype == FDC_BF16)
      FDC_LAUNCH_TILES(decode_tiles_kernel<uint16_t>, heads, wtiles, static_cast<const float*>(q_lat),
                       static_cast<const uint16_t*>(k_cache), static_cast<const uint16_t*>(v_cache), scale_log2,
                       static_cast<float*>(o_lat), partials, W, planned, lens);
    else if (lay->dtype == FDC_FP8)
      FDC_LAUNCH_TILES(decode_tiles_kernel<uint8_t>, heads, wtiles, static_cast<const float*>(q_lat),
                       static_cast<const uint8_t*>(k_cache), static_cast<const uint8_t*>(v_cache), scale_log2,
                       static_cast<float*>(o_lat), partials, W, planned, lens);
    else if (lay->dtype == FDC_FP4)
      FDC_LAUNCH_TILES(decode_tiles_kernel<fp4_t>, heads, wtiles, static_cast<const float*>(q_lat),
                       static_cast<const fp4_t*>(k_cache), static_cast<const fp4_t*>(v_cache), scale_log2,
                       static_cast<float*>(o_lat), partials, W, planned, lens);
    else
      FDC_LAUNCH_TILES(decode_tiles_kernel<float>, heads, wtiles, static_cast<const float*>(q_lat),
                       static_cast<const float*>(k_cache), static_cast<const float*>(v_cache), scale_log2,
                       static_cast<float*>(o_lat), partials, W, planned, lens);
#undef FDC_LAUNCH_TILES
    FDC_HIP_CHECK(hipGetLastError());
  }
  // One rule for every plan, so that a result does not depend on where the plan was made: a unit of at most
  // kMergeWaveMax tiles is merged by one wavefront in slot order, a unit of more by sixteen. Each kernel skips
  // the other's units. A host plan knows which kinds it has; for a device plan the host only knows how many
  // granules a sequence can hold.
  const bool any_wide = plan->on_device ? plan->max_unit_granules > kMergeWaveMax : plan->max_items_per_unit > kMergeWaveMax;
  const bool any_wave = plan->on_device || plan->min_items_per_unit <= kMergeWaveMax;
  if (any_wave)
    hipLaunchKernelGGL(decode_merge_wave_kernel, dim3((plan->n_merge_units + kMergeWaves - 1) / kMergeWaves),
                       dim3(kMergeWaves * 64), 0, st, units, partials, static_cast<float*>(o_lat), plan->n_merge_units);
  if (any_wide)
    hipLaunchKernelGGL(decode_merge_wide_kernel, dim3(plan->n_merge_units), dim3(kWideWaves * 64), 0, st, units, partials,
                       static_cast<float*>(o_lat));
  FDC_HIP_CHECK(hipGetLastError());
  return FDC_OK;
}

extern "C" {

fdc_status fdc_latent_attn_decode(const fdc_layout* lay, const fdc_plan* plan, const void* q_lat, const void* k_cache,
                                  const void* v_cache, float scale, void* o_lat, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  return decode_impl(lay, plan, nullptr, q_lat, k_cache, v_cache, scale, o_lat, workspace, workspace_bytes, stream);
}

fdc_status fdc_latent_attn_decode_static(const fdc_layout* lay, const fdc_plan* plan, const void* q_lat,
                                         const void* k_cache, const void* v_cache, float scale, void* o_lat,
                                         void* stream) {
  struct DropProfileRequest {   // a pending profiling request belongs to this call even if it fails before the launch
    bool armed = true;
    ~DropProfileRequest() {
      if (armed) g_prof_start = g_prof_stop = nullptr;
    }
  } drop;
  if (!lay || !plan) FDC_FAIL(FDC_INVALID_ARG, "fdc_latent_attn_decode_static: NULL argument");
  if (plan->kind != 0 || plan->lay != lay)
    FDC_FAIL(FDC_INVALID_ARG, "fdc_latent_attn_decode_static: not a decode plan of this layout");
  if (plan->on_device)
    FDC_FAIL(FDC_INVALID_ARG, "fdc_latent_attn_decode_static: plans made on the device keep their tables in the "
                              "caller's workspace; use fdc_latent_attn_decode");
  if (plan->workspace_bytes > kStaticScratchBytes)
    FDC_FAIL(FDC_WORKSPACE_TOO_SMALL, "fdc_latent_attn_decode_static: the plan needs %zu bytes of workspace, the "
                                      "built-in one has %zu", plan->workspace_bytes, kStaticScratchBytes);
  int dev = 0;
  FDC_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) FDC_FAIL(FDC_INVALID_ARG, "fdc_latent_attn_decode_static: device %d", dev);
  void* ws = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    ScratchOfDevice& sd = g_scratch_of[dev];
    if (!sd.ptr) {
      void* p = nullptr;
      FDC_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
      if (!p || (reinterpret_cast<uintptr_t>(p) & 255u) != 0)
        FDC_FAIL(FDC_HIP_ERROR, "fdc_latent_attn_decode_static: bad address %p for the built-in workspace", p);
      sd.ptr = p;
    }
    ws = sd.ptr;
    if (sd.resident_plan != plan->serial) {   // tables of another plan (or none) are in the array: replace them
      sd.resident_plan = 0;
      FDC_HIP_CHECK(hipMemcpyAsync(ws, plan->image.data(), plan->image.size(), hipMemcpyHostToDevice,
                                   static_cast<hipStream_t>(stream)));
      sd.resident_plan = plan->serial;
    }
  }
  // The partial states need no clearing: the tile kernel writes every slot the merge reads.
  drop.armed = false;
  return decode_impl(lay, plan, nullptr, q_lat, k_cache, v_cache, scale, o_lat, ws, kStaticScratchBytes, stream);
}

fdc_status fdc_latent_attn_decode_at(const fdc_layout* lay, const fdc_plan* plan, const int32_t* seq_len,
                                     const void* q_lat, const void* k_cache, const void* v_cache, float scale,
                                     void* o_lat, void* workspace, size_t workspace_bytes, void* stream) {
  if (!seq_len) FDC_FAIL(FDC_INVALID_ARG, "fdc_latent_attn_decode_at: seq_len is NULL");
  return decode_impl(lay, plan, seq_len, q_lat, k_cache, v_cache, scale, o_lat, workspace, workspace_bytes, stream);
}

}  // extern "C"
