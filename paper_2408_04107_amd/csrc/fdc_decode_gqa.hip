// Grouped-query decode attention on the latent cache (Section 5.1, GQA paragraph; Section 5 step 7):
// g query heads share the K' / V' rows of one key/value head, so a tile of that head is streamed
// from HBM once and serves the whole group.
//
// Design for gfx950. With g queries per cached row the per-row work no longer fits the vector ALU
// at stream speed (one multiply-add per element AND query), but it is exactly what the matrix core
// does: the group is a 16-row operand (g <= 16, padded with zero rows). As in the prefill kernel
// both products are computed transposed,
//     S^T = K' Q'^T       (A = 16 cached rows x 32 k,  B = the 16 query rows)     v_mfma_f32_16x16x32_bf16
//     O^T = V'^T P^T      (A = V'^T,                   B = P^T, k = 32 tokens)
// so a lane owns ONE query (column l % 16): the score tile is already the operand of the second
// product and the softmax state lives in the lanes that use it. A worker is one wavefront, as in the
// multi-head decode kernel, and takes the same tiles from the same planner.
//   K': the A operand of the first product is read straight from global memory in its MFMA layout
//       (lane (l%16, l/16) loads the 16 bytes at row l%16, k = 32 ks + 8 (l/16)): no LDS, no shuffle.
//   V': needs a transpose (the contraction runs over tokens). Its rows are loaded as one contiguous
//       span, 16 bytes per lane, written unchanged to a wave-private LDS region and read back with
//       the transposing LDS load (ds_read_b64_tr_b16). No workgroup barrier anywhere: LDS operations
//       of one wave execute in order.
// A step covers 32 * NB tokens, NB chosen per rank class so that a step is about 16 KiB of cache;
// the K' registers are refilled for the next step as soon as the scores are out and the V' registers
// as soon as they are in LDS, every load unconditional (the raw-buffer range check returns zeros
// past the tile's end). Results go to the same partial-state slots / outputs as the multi-head
// kernel, one per query head, and the same merge kernel combines them.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>

#include "fdc_internal.h"

namespace fdc {

typedef __bf16 gq_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 gq_bf16x2 __attribute__((ext_vector_type(2)));
typedef float gq_f32x2 __attribute__((ext_vector_type(2)));
typedef float gq_f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t gq_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t gq_u32x2 __attribute__((ext_vector_type(2)));
typedef short gq_s16x4 __attribute__((ext_vector_type(4)));

constexpr int kGqaWaves = kWorkersPerGroup;  // workers (wavefronts) per workgroup
constexpr int kGqaLdsElems = 4096;       // bf16 elements of V' staging per wave (8 KiB)
constexpr float kGqaLog2e = 1.4426950408889634f;
constexpr float kGqaRaise = 6.0f;        // lazy softmax reference: p <= 2^6 between raises
constexpr int kGqaStream = 2;            // "nt" cache policy of the K'/V' stream (read once)

union GqFrag {
  gq_u32x4 u;
  gq_bf16x8 v;
};

__device__ __forceinline__ uint32_t gq_pack(float lo, float hi) {  // v_cvt_pk_bf16_f32
  union { gq_bf16x2 v; uint32_t u; } r;
  r.v = __builtin_convertvector(gq_f32x2{lo, hi}, gq_bf16x2);
  return r.u;
}
// Sixteen E4M3 codes (16 bytes) -> sixteen bf16 in the same order: v_cvt_scalef32_pk_bf16_fp8 with scale 1
// turns two codes into two packed bf16 in one instruction (bf16 holds every code value exactly).
__device__ __forceinline__ uint32_t gq_codes_to_bf16(uint32_t word, bool upper) {
  union { gq_bf16x2 v; uint32_t u; } r;
  r.v = upper ? __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(word, 1.0f, true)
              : __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(word, 1.0f, false);
  return r.u;
}
__device__ __forceinline__ void gq_widen16(const gq_u32x4& c, gq_u32x4& lo, gq_u32x4& hi) {
  lo = gq_u32x4{gq_codes_to_bf16(c[0], false), gq_codes_to_bf16(c[0], true), gq_codes_to_bf16(c[1], false),
                gq_codes_to_bf16(c[1], true)};
  hi = gq_u32x4{gq_codes_to_bf16(c[2], false), gq_codes_to_bf16(c[2], true), gq_codes_to_bf16(c[3], false),
                gq_codes_to_bf16(c[3], true)};
}
// reductions over the four lanes l, l ^ 16, l ^ 32, l ^ 48 that share a query
__device__ __forceinline__ float gq_row_max(float v) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float gq_row_sum(float v) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}
__device__ __forceinline__ void gq_lds_order() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// M = ceil(max(rk, rv) / 32) in 1..4. Loop bounds are compile-time in M; the actual ranks only
// guard (wave-uniformly) the steps a narrower side does not need.
// TC is the cache element: uint16_t (bf16) or uint8_t (E4M3 codes). Codes are widened to bf16 (exact)
// in registers: a 16-byte load then holds sixteen k of its row, i.e. the operands of TWO MFMA steps, so
// the k index is permuted (step 2 b + h takes elements 64 b + 16 lg + 8 h .. + 8 of lane row lg); Q' is
// laid out the same way, and a product does not depend on the order of its terms' index.
template <int M, typename TC>
__device__ __forceinline__ void gqa_tile(const DecTile& td, const float* __restrict__ q_lat,
                                         const TC* __restrict__ kc, const TC* __restrict__ vc,
                                         float scale_log2, float* __restrict__ o_lat, float* __restrict__ partials,
                                         uint16_t* lds, int lane) {
  constexpr int NB = M == 1 ? 4 : (M == 2 ? 2 : 1);  // 32-token sub-blocks per step
  constexpr int BT = 32 * NB;
  constexpr int ES = (int)sizeof(TC);                // bytes per cached element
  constexpr int MB = (M + 1) / 2;                    // E4M3: 64-element blocks of a K' row (two MFMA steps each)
  constexpr int KS = ES == 2 ? M : 2 * MB;           // MFMA k-steps of the score product
  constexpr int KL = ES == 2 ? M : MB;               // 16-byte K' loads per 16-token half
  constexpr int NVL = ES == 2 ? NB * 2 * M : NB * M; // most 1 KiB loads a step of V' can need
  static_assert(BT * 32 * M <= kGqaLdsElems, "V' staging region");
  const int rk = td.rk_rv & 0xffff, rv = td.rk_rv >> 16;
  const int rk32 = (rk + 31) / 32, rv16 = rv / 16;
  const int ln = lane % 16, lg = lane / 16;
  const int g = td.g, len = td.len;
  const uint32_t rk2 = (uint32_t)rk * ES, rv2 = (uint32_t)rv * ES;   // bytes per cached row
  constexpr uint32_t kOob = 0x80000000u;

  // Q' operand: lane (ln, lg) holds k = 32 ks + 8 lg .. + 8 of query ln (zero rows past the group).
  // q' arrives in fp32 and a bf16 operand keeps 8 bits of it, which alone would put the scores of a
  // peaked softmax outside the output tolerance; so q' = qf + ql with qf = bf16(q') and
  // ql = bf16(q' - qf) (16 bits together), and the score product is taken with both. The matrix
  // core is idle most of the time in this kernel (the stream is the limit), the second product is free.
  GqFrag qf[KS], ql[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const int col = ES == 2 ? 32 * ks + 8 * lg : 64 * (ks / 2) + 16 * lg + 8 * (ks % 2);
    if (ln < g && col < rk) {
      const float* qp = q_lat + td.q_elem + ln * rk + col;
      const float4 a = *reinterpret_cast<const float4*>(qp), b = *reinterpret_cast<const float4*>(qp + 4);
      const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
      float r[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t hi = gq_pack(v[2 * e], v[2 * e + 1]);
        qf[ks].u[e] = hi;
        r[2 * e] = v[2 * e] - __uint_as_float(hi << 16);
        r[2 * e + 1] = v[2 * e + 1] - __uint_as_float(hi & 0xffff0000u);
      }
      ql[ks].u = gq_u32x4{gq_pack(r[0], r[1]), gq_pack(r[2], r[3]), gq_pack(r[4], r[5]), gq_pack(r[6], r[7])};
    } else {
      qf[ks].u = gq_u32x4{0, 0, 0, 0};
      ql[ks].u = gq_u32x4{0, 0, 0, 0};
    }
  }

  const __amdgpu_buffer_rsrc_t k_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<TC*>(kc + td.k_elem), 0, (int)(len * rk2), 0x00020000);
  const __amdgpu_buffer_rsrc_t v_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<TC*>(vc + td.v_elem), 0, (int)(len * rv2), 0x00020000);
  // K' load (nb, j, kl): row tok0 + 32 nb + 16 j + ln, bytes 64 kl + 16 lg of the row (bf16: the fragment
  // of step kl; E4M3: the sixteen codes of steps 2 kl and 2 kl + 1)
  uint32_t kcol[KL];
#pragma unroll
  for (int kl = 0; kl < KL; ++kl) kcol[kl] = (64 * kl + 16 * lg < (int)rk2) ? (uint32_t)(64 * kl + 16 * lg) : kOob;
  const uint32_t vlane = (uint32_t)lane * 16;
  // 1 KiB loads of a step's V' span: 32 NB tokens x rv elements (a last half load of an E4M3 span also
  // brings rows of the next step; they land inside the staging region and are never read)
  const int n_vl = ES == 2 ? NB * rv16 : (NB * rv16 + 1) / 2;

  gq_u32x4 kreg[NB][2][KL], vreg[NVL];
  auto fetch_k = [&](int tok0) {
    const uint32_t row = (uint32_t)(tok0 + ln) * rk2;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int kl = 0; kl < KL; ++kl)
          kreg[nb][j][kl] = __builtin_amdgcn_raw_buffer_load_b128(
              k_rsrc, (int)(kcol[kl] + row + (uint32_t)(32 * nb + 16 * j) * rk2), 0, kGqaStream);
  };
  auto fetch_v = [&](int tok0) {
    const uint32_t base = (uint32_t)tok0 * rv2 + vlane;
#pragma unroll
    for (int i = 0; i < NVL; ++i)
      vreg[i] = __builtin_amdgcn_raw_buffer_load_b128(v_rsrc, (int)(i < n_vl ? base + (uint32_t)i * 1024u : kOob), 0,
                                                      kGqaStream);
  };

  gq_f32x4 oacc[2 * M];
#pragma unroll
  for (int c = 0; c < 2 * M; ++c) oacc[c] = gq_f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;   // of query ln, over the tokens this lane sees

  fetch_k(0);
  fetch_v(0);
  for (int tok0 = 0; tok0 < len; tok0 += BT) {
    // scores: st[nb][j] = tokens tok0 + 32 nb + 16 j + 4 lg + e of query ln
    gq_f32x4 st[NB][2];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        GqFrag kf;
        if constexpr (ES == 2) {
          kf.u = kreg[nb][j][0];
          st[nb][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf.v, ql[0].v, gq_f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
          st[nb][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf.v, qf[0].v, st[nb][j], 0, 0, 0);
#pragma unroll
          for (int ks = 1; ks < M; ++ks) {
            if (ks >= rk32) break;
            kf.u = kreg[nb][j][ks];
            st[nb][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf.v, ql[ks].v, st[nb][j], 0, 0, 0);
            st[nb][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf.v, qf[ks].v, st[nb][j], 0, 0, 0);
          }
        } else {
          st[nb][j] = gq_f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int kl = 0; kl < KL; ++kl) {
            if (64 * kl >= rk) break;
            gq_u32x4 lo, hi;
            gq_widen16(kreg[nb][j][kl], lo, hi);
            kf.u = lo;
            st[nb][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf.v, ql[2 * kl].v, st[nb][j], 0, 0, 0);
            st[nb][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf.v, qf[2 * kl].v, st[nb][j], 0, 0, 0);
            kf.u = hi;
            st[nb][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf.v, ql[2 * kl + 1].v, st[nb][j], 0, 0, 0);
            st[nb][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf.v, qf[2 * kl + 1].v, st[nb][j], 0, 0, 0);
          }
        }
      }
    __builtin_amdgcn_sched_barrier(0);
    fetch_k(tok0 + BT);   // the K' registers are free again
    __builtin_amdgcn_sched_barrier(0);

    if (tok0 + BT > len) {   // last step of the tile: tokens past its end
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (tok0 + 32 * nb + 16 * j + 4 * lg + e >= len) st[nb][j][e] = -INFINITY;
    }
    float mx = -INFINITY;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) mx = fmaxf(mx, st[nb][j][e]);
    // raise the reference of a query only when some lane beats it by kGqaRaise (log2 units)
    if (__any(mx * scale_log2 > m_run * scale_log2 + kGqaRaise)) {
      mx = gq_row_max(mx);
      const float m_new = fmaxf(m_run, mx);
      const float m_ref = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_ref) * scale_log2);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int c = 0; c < 2 * M; ++c) oacc[c] *= alpha;
    }
    const float neg = m_run == -INFINITY ? 0.f : -m_run * scale_log2;
    GqFrag pf[NB];
    float psum = 0.f;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      float p[2][4];
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          p[j][e] = __builtin_amdgcn_exp2f(fmaf(st[nb][j][e], scale_log2, neg));
          psum += p[j][e];
        }
      pf[nb].u = gq_u32x4{gq_pack(p[0][0], p[0][1]), gq_pack(p[0][2], p[0][3]), gq_pack(p[1][0], p[1][1]),
                          gq_pack(p[1][2], p[1][3])};
    }
    l_run += psum;

    // V' rows of the step: registers -> LDS, unchanged order (row-major, pitch rv)
    gq_lds_order();   // the previous step's transposing reads come first
#pragma unroll
    for (int i = 0; i < NVL; ++i)
      if (i < n_vl) {
        if constexpr (ES == 2) {
          *reinterpret_cast<gq_u32x4*>(&lds[(i * 64 + lane) * 8]) = vreg[i];
        } else {   // sixteen codes -> sixteen bf16, same row-major order
          gq_u32x4 lo, hi;
          gq_widen16(vreg[i], lo, hi);
          *reinterpret_cast<gq_u32x4*>(&lds[(i * 64 + lane) * 16]) = lo;
          *reinterpret_cast<gq_u32x4*>(&lds[(i * 64 + lane) * 16 + 8]) = hi;
        }
      }
    __builtin_amdgcn_sched_barrier(0);
    fetch_v(tok0 + BT);   // the V' registers are free again
    __builtin_amdgcn_sched_barrier(0);
    gq_lds_order();

    // O^T += V'^T P^T. A operand: lane (ln, lg) holds column 16 c + ln of tokens 32 nb + 4 lg + e and
    // 32 nb + 16 + 4 lg + e (the order P has them). Transposing load: inside the 16-lane group lg,
    // source lane s addresses token 4 lg + s / 4, columns 16 c + 4 (s % 4) ..
    const uint16_t* vsrc = lds + (4 * lg + ln / 4) * rv + 4 * (ln % 4);
#pragma unroll
    for (int c = 0; c < 2 * M; ++c) {
      if (c >= rv16) break;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const uint16_t* a0 = vsrc + (32 * nb) * rv + 16 * c;
        union { gq_s16x4 s; gq_u32x2 u; } lo, hi;
        lo.s = __builtin_amdgcn_ds_read_tr16_b64_v4i16((gq_s16x4 __attribute__((address_space(3)))*)(a0));
        hi.s = __builtin_amdgcn_ds_read_tr16_b64_v4i16((gq_s16x4 __attribute__((address_space(3)))*)(a0 + 16 * rv));
        GqFrag vf;
        vf.u = gq_u32x4{lo.u[0], lo.u[1], hi.u[0], hi.u[1]};
        oacc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf.v, pf[nb].v, oacc[c], 0, 0, 0);
      }
    }
  }

  // tile result of query ln: lane (ln, lg) holds O[16 c + 4 lg + e]
  const float l = gq_row_sum(l_run);
  if (ln < g) {
    if (td.slot < 0) {
      const float inv = 1.f / l;
      float* o = o_lat + td.o_elem + ln * rv + 4 * lg;
#pragma unroll
      for (int c = 0; c < 2 * M; ++c) {
        if (c >= rv16) break;
        *reinterpret_cast<float4*>(o + 16 * c) = float4{oacc[c][0] * inv, oacc[c][1] * inv, oacc[c][2] * inv, oacc[c][3] * inv};
      }
    } else {
      float* pp = partials + (int64_t)(td.slot + ln * td.slot_stride) * kPartialStride;
#pragma unroll
      for (int c = 0; c < 2 * M; ++c) {
        if (c >= rv16) break;
        *reinterpret_cast<float4*>(pp + 4 + 16 * c + 4 * lg) = float4{oacc[c][0], oacc[c][1], oacc[c][2], oacc[c][3]};
      }
      if (lg == 0) pp[0] = m_run * scale_log2, pp[1] = l;
    }
  }
}

template <typename TC>
__global__ __launch_bounds__(kGqaWaves * 64) void decode_gqa_tiles_kernel(
    const DecWorker* __restrict__ workers, const DecTile* __restrict__ wtiles, const float* __restrict__ q_lat,
    const TC* __restrict__ kc, const TC* __restrict__ vc, float scale_log2, float* __restrict__ o_lat,
    float* __restrict__ partials, int n_workers, const int32_t* __restrict__ planned_len,
    const int32_t* __restrict__ seq_len) {
  __shared__ __attribute__((aligned(16))) uint16_t lds_all[kGqaWaves][kGqaLdsElems];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
  const int lane = threadIdx.x % 64;
  const int worker = blockIdx.x * kGqaWaves + wave;
  if (worker >= n_workers) return;
  uint16_t* lds = lds_all[wave];
  const DecWorker* hd = workers + worker;
  const int count = hd->count, begin = hd->begin;
  if (count == 0) return;
  DecTile td = hd->first;
  for (int i = 0;;) {
    const DecTile next = wtiles[begin + min(i + 1, count - 1)];   // requested ahead of the tile boundary
    td.len = dec_tile_len(td, planned_len, seq_len);
    const int rmax = max(td.rk_rv & 0xffff, td.rk_rv >> 16);
    switch ((rmax + 31) / 32) {
      case 1: gqa_tile<1, TC>(td, q_lat, kc, vc, scale_log2, o_lat, partials, lds, lane); break;
      case 2: gqa_tile<2, TC>(td, q_lat, kc, vc, scale_log2, o_lat, partials, lds, lane); break;
      case 3: gqa_tile<3, TC>(td, q_lat, kc, vc, scale_log2, o_lat, partials, lds, lane); break;
      case 4: gqa_tile<4, TC>(td, q_lat, kc, vc, scale_log2, o_lat, partials, lds, lane); break;
      default: break;
    }
    if (++i >= count) break;
    td = next;
  }
}

fdc_status decode_gqa_workers_per_cu(int* waves) {
  int nb = 0;
  FDC_HIP_CHECK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, decode_gqa_tiles_kernel<uint16_t>, kGqaWaves * 64, 0));
  *waves = std::max(nb, 1) * kGqaWaves;
  return FDC_OK;
}

fdc_status launch_decode_gqa(const DecWorker* heads, const DecTile* wtiles, const float* q_lat, const void* kc,
                             const void* vc, bool e4m3, float scale, float* o_lat, float* partials, int n_workers,
                             const int32_t* planned_len, const int32_t* seq_len, hipEvent_t ev0, hipEvent_t ev1,
                             hipStream_t st) {
  const dim3 grid((n_workers + kGqaWaves - 1) / kGqaWaves), block(kGqaWaves * 64);
  const float scale_log2 = scale * kGqaLog2e;
  // ev0 / ev1 (both or neither): events of the kernel's own dispatch, for the caller's profiling request
  if (e4m3) {
    const uint8_t* k8 = static_cast<const uint8_t*>(kc);
    const uint8_t* v8 = static_cast<const uint8_t*>(vc);
    if (ev0)
      hipExtLaunchKernelGGL(decode_gqa_tiles_kernel<uint8_t>, grid, block, 0, st, ev0, ev1, 0, heads, wtiles, q_lat, k8, v8,
                            scale_log2, o_lat, partials, n_workers, planned_len, seq_len);
    else
      hipLaunchKernelGGL(decode_gqa_tiles_kernel<uint8_t>, grid, block, 0, st, heads, wtiles, q_lat, k8, v8, scale_log2,
                         o_lat, partials, n_workers, planned_len, seq_len);
  } else {
    const uint16_t* k16 = static_cast<const uint16_t*>(kc);
    const uint16_t* v16 = static_cast<const uint16_t*>(vc);
    if (ev0)
      hipExtLaunchKernelGGL(decode_gqa_tiles_kernel<uint16_t>, grid, block, 0, st, ev0, ev1, 0, heads, wtiles, q_lat, k16,
                            v16, scale_log2, o_lat, partials, n_workers, planned_len, seq_len);
    else
      hipLaunchKernelGGL(decode_gqa_tiles_kernel<uint16_t>, grid, block, 0, st, heads, wtiles, q_lat, k16, v16, scale_log2,
                         o_lat, partials, n_workers, planned_len, seq_len);
  }
  FDC_HIP_CHECK(hipGetLastError());
  return FDC_OK;
}

}  // namespace fdc
