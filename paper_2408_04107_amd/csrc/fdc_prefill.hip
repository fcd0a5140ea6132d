// Causal prefill attention on the latent cache (Section 5, step 7; Section 5.3 prefill: Q-block
// tasks of equalised cost handed to workers).
//
// Design for gfx950. A worker is one workgroup of sixteen waves; it walks the Q-block tasks the
// planner gave it. A task is processed in passes of 256 query rows, 16 rows (one MFMA tile) per
// wave. K' and V' blocks of 128 tokens are staged through LDS once per workgroup, both row-major
// as they sit in the cache (K' with its rank zero-padded to a multiple of 32), in two
// alternating buffers so that a block costs one barrier; a wave works through a block as two sets
// of 64 tokens (one softmax update each). Against 128-row passes and 64-token blocks (eight waves,
// two workgroups per compute unit: the same 4 waves per SIMD and the same registers) every cached
// row is staged half as often, there are half as many barriers per token, and the register
// prefetch of the next block has twice as long to arrive: 8-10 % faster at every rank.
// All products are transposed ones,
//     S^T = K' Q'^T          (A = K' rows,   B = Q' rows)      v_mfma_f32_16x16x32_bf16
//     O^T = V'^T P^T         (A = V'^T rows, B = P^T)          v_mfma_f32_16x16x32_bf16
// because then every quantity a lane holds belongs to ONE query row (column l%16 of the MFMA
// output): the score tile comes out of the first product already in the operand layout of the
// second (no LDS round trip for P), the running max / sum live in the lanes that use them, and
// the rescale of O needs no cross-lane traffic. The V'^T operand is read from the row-major tile
// with the transposing LDS load of gfx950 (ds_read_b64_tr_b16): inside a group of 16 lanes, lane s
// supplies the address of 4 consecutive columns of token s/4, and lane L receives column L of the
// four tokens. The k index of the second product (tokens) is spread over lanes in the order the
// first product delivers it; both operands use the same order.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "fdc_internal.h"

namespace fdc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int QT = 1;                    // 16-row MFMA tiles of queries per wave
constexpr int BC = 64;                   // tokens per score tile set (one softmax update)
constexpr int NH = 2;                    // score tile sets per staged block
constexpr int BCB = BC * NH;             // tokens per staged K'/V' block (one barrier)
static_assert(BCB == kPrefillBlockTokens, "a page of a paged cache holds whole staged blocks");
constexpr int kRowsPerWave = 16 * QT;
constexpr int kRowsPerPass = 256;         // query rows a workgroup works on at a time (sixteen waves)
constexpr int kPreThreads = 64 * (kRowsPerPass / kRowsPerWave);
constexpr int kPreWavesPerSimd = kPreThreads / 256 * (160 * 1024 / (2 * BCB * (144 + 144) * 2));  // workgroups that fit the LDS
// LDS row lengths in elements. A 16-byte LDS read serves 16 lanes per pass, and (measured with two
// active lanes at a time) the passes are not the four lane rows: lanes {0-3, 12-15, 20-27} share one,
// {4-11, 16-19, 28-31} the next, and the upper half mirrors that. For the K' fragment read (lane
// (ln, lg) takes 16 bytes of row ln at column chunk lg) a pass therefore holds eight rows at chunk
// lg and the other eight at chunk lg + 1. A row stride of 2 (mod 16) chunks puts the first group on
// the even 16-byte bank groups and the second on the odd ones: no conflicts, where the 272-byte
// stride that would suit lane-row passes gave a two-way conflict on every read (counter ratio 0.50).
constexpr int KROW = 128 + 16;           // K' tile: 288 bytes = 18 chunks
constexpr int VROW = 128 + 16;           // V' tile: 288 bytes (the transposing 8-byte reads are conflict free too)
constexpr int kStageElems = BCB * KROW + BCB * VROW;  // one buffer: K' tile then V' tile
constexpr float kLog2eP = 1.4426950408889634f;
constexpr float kRaise = 5.0f;           // lazy softmax reference: p <= 2^5 between raises
// (the k-steps ceil(rk / 32) <= 4 of the score product and the column tiles rv / 16 <= 8 of the output are
// template parameters of the task body: an upper bound of the head's own counts)

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {  // v_cvt_pk_bf16_f32, round to nearest even
  union { bf16x2 v; uint32_t u; } r;
  r.v = __builtin_convertvector(f32x2{lo, hi}, bf16x2);
  return r.u;
}

// Reductions over the four lanes l, l ^ 16, l ^ 32, l ^ 48 that share a query row, with the lane
// swaps of gfx950 (v_permlane16_swap exchanges the odd 16-lane rows of its first operand with the
// even rows of its second, v_permlane32_swap the upper half of the first with the lower half of
// the second), which stay in the vector ALU instead of going through LDS like a generic shuffle.
__device__ __forceinline__ float row_max(float v) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float row_sum(float v) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

union Frag {
  u32x4 u;
  bf16x8 v;
};

// The two products of a 64-token set, with the number of k-steps / column tiles as a compile-time
// constant (the caller switches on the head's rank class). With run-time bounds the unrolled loops
// kept a branch after every step, so each LDS read sat in a basic block of its own right in front
// of the multiply that needs it and its whole latency was exposed, step after step. Here a
// fragment is requested as soon as the multiply that used its registers has been issued, one tile
// ahead, so the reads of tile j + 1 are in flight under the multiplies of tile j.
template <int RK32T, int NQ>
__device__ __forceinline__ void score_tiles(const uint16_t* __restrict__ lk, const Frag (*qf)[RK32T], f32x4 (*st)[NQ], int ln, int lg) {
  Frag kf[RK32T];
  const uint16_t* src = lk + ln * KROW + 8 * lg;
#pragma unroll
  for (int ks = 0; ks < RK32T; ++ks) kf[ks].u = *reinterpret_cast<const u32x4*>(src + 32 * ks);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
#pragma unroll
    for (int ks = 0; ks < RK32T; ++ks) {
      const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < NQ; ++i)
        st[j][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks].v, qf[i][ks].v, ks == 0 ? zero : st[j][i], 0, 0, 0);
      if (j < 3) kf[ks].u = *reinterpret_cast<const u32x4*>(src + 16 * (j + 1) * KROW + 32 * ks);
    }
  }
}

// O^T += V'^T P^T for RV16T column tiles. A operand: lane (ln, lg) must hold column 16 c + ln for the
// tokens 32 jp + 4 lg + e and 32 jp + 16 + 4 lg + e (the order P has them). Transposing load: inside
// the 16-lane group lg, source lane s addresses token 4 lg + s / 4, columns 16 c + 4 (s % 4) ..
template <int RV16T, int NQ>
__device__ __forceinline__ void pv_tiles(const uint16_t* __restrict__ lv, const Frag (*pf)[2], f32x4 (*oacc)[RV16T], int ln, int lg) {
  const uint16_t* vsrc = lv + (4 * lg + ln / 4) * VROW + 4 * (ln % 4);
  auto load = [&](int idx) {
    const uint16_t* a0 = vsrc + (32 * (idx % 2)) * VROW + 16 * (idx / 2);
    union { s16x4 s; u32x2 u; } lo, hi;
    lo.s = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(a0));
    hi.s = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(a0 + 16 * VROW));
    Frag f;
    f.u = u32x4{lo.u[0], lo.u[1], hi.u[0], hi.u[1]};
    return f;
  };
  Frag vf[2];
  vf[0] = load(0);
#pragma unroll
  for (int idx = 0; idx < 2 * RV16T; ++idx) {
    if (idx + 1 < 2 * RV16T) vf[(idx + 1) & 1] = load(idx + 1);
#pragma unroll
    for (int i = 0; i < NQ; ++i)
      oacc[i][idx / 2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[idx & 1].v, pf[i][idx % 2].v, oacc[i][idx / 2], 0, 0, 0);
  }
}

// The body of a task is instantiated per rank class (RK32 = k-steps of the score product, RV16 = column
// tiles of the output, the head's own counts or the next instantiated ones above): loop bounds are
// compile-time, so the products are straight-line code with their LDS reads pipelined, and the
// accumulators of a narrow head take the registers that head needs and no more. The kernel switches
// per task; a workgroup runs one instantiation at a time.
// TC is the cache element: uint16_t (bf16) or uint8_t (E4M3 codes, widened to bf16, which holds them
// exactly, on their way from the staging registers to LDS; everything after that is the same).
template <typename TC, int RK32, int RV16>
__device__ __forceinline__ void prefill_task(const PreTask& t, const uint16_t* __restrict__ q_lat,
                                             const TC* __restrict__ kc, const TC* __restrict__ vc,
                                             float scale_log2, int causal, uint16_t* __restrict__ o_lat,
                                             const int32_t* __restrict__ page_table, int64_t page_stride_k,
                                             int64_t page_stride_v, uint16_t* lds) {
  const int rk = t.rk_rv & 0xffff, rv = t.rk_rv >> 16;
  const int rk32 = (rk + 31) / 32, rv16 = rv / 16;
  const int RKP = rk32 * 32;  // rank of the K' rows in LDS, padded with zeros
  const int tid = threadIdx.x, lane = tid % 64;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);   // known uniform: conditions on it become scalar branches
  const int ln = lane % 16, lg = lane / 16;
  // cache element: bf16 (TC = uint16_t), an E4M3 code (uint8_t) or an E2M1 code (fp4_t: two per byte). A staging
  // chunk is what a lane loads at once: 16 bytes, 8 for E2M1 (sixteen codes, so that the narrowest row is a chunk)
  constexpr bool kFp4 = sizeof(TC) == 1 && !std::is_same<TC, uint8_t>::value;
  constexpr int BITS = kFp4 ? 4 : 8 * (int)sizeof(TC);
  constexpr int CB = kFp4 ? 8 : 16;     // bytes per chunk
  constexpr int EPC = CB * 8 / BITS;    // elements per chunk
  const uint8_t* kbase = reinterpret_cast<const uint8_t*>(kc) + t.k_elem * BITS / 8;
  const uint8_t* vbase = reinterpret_cast<const uint8_t*>(vc) + t.v_elem * BITS / 8;

  // zero the rank padding of both K' tiles once: staging never writes those columns
  if (RKP != rk) {
    for (int i = tid; i < 2 * BCB * (RKP - rk); i += kPreThreads) {
      const int buf = i / (BCB * (RKP - rk)), j = i % (BCB * (RKP - rk));
      lds[buf * kStageElems + (j / (RKP - rk)) * KROW + rk + j % (RKP - rk)] = 0;
    }
  }

  // staging map: a token row of rank r is r / EPC chunks of 16 bytes (r / 8 for bf16); thread tid takes chunk
  // tid % (r/8) of row tid / (r/8), so every lane of a sweep carries data whatever the rank (one
  // division per task). A sweep covers kPreThreads / (r/8) >= 32 rows: one sweep per block for
  // ranks <= 64, two above. K' and V' have their own maps (rk != rv).
  constexpr int kSweeps = 2;
  const int lpk = rk / EPC, lpv = rv / EPC;
  const int k_rps = kPreThreads / lpk, v_rps = kPreThreads / lpv;
  const int k_row = tid / lpk, k_cc = tid - k_row * lpk;
  const int v_row = tid / lpv, v_cc = tid - v_row * lpv;
  const int k_sweeps = (BCB + k_rps - 1) / k_rps, v_sweeps = (BCB + v_rps - 1) / v_rps;
  // the unit's K' and V' rows [0, kv_len) as raw buffers (at most 131072 * 256 bytes each)
  const __amdgpu_buffer_rsrc_t k_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(kbase), 0, t.kv_len * rk * BITS / 8, 0x00020000);
  const __amdgpu_buffer_rsrc_t v_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(vbase), 0, t.kv_len * rv * BITS / 8, 0x00020000);
  // per sweep: byte offset of the lane's chunk in block 0 (out of range when the lane has no row)
  // and its LDS element offset
  uint32_t k_goff[kSweeps], v_goff[kSweeps];
  int k_loff[kSweeps], v_loff[kSweeps];
  bool k_on[kSweeps], v_on[kSweeps];
#pragma unroll
  for (int i = 0; i < kSweeps; ++i) {
    const int kr = k_row + i * k_rps, vr = v_row + i * v_rps;
    k_on[i] = k_row < k_rps && kr < BCB;
    v_on[i] = v_row < v_rps && vr < BCB;
    k_goff[i] = k_on[i] ? (uint32_t)(kr * rk * BITS / 8 + k_cc * CB) : 0x80000000u;
    v_goff[i] = v_on[i] ? (uint32_t)(vr * rv * BITS / 8 + v_cc * CB) : 0x80000000u;
    k_loff[i] = kr * KROW + k_cc * EPC;
    v_loff[i] = vr * VROW + v_cc * EPC;
  }

  for (int r0 = 0; r0 < t.rows; r0 += kRowsPerPass) {
    const int pass_rows = min(kRowsPerPass, t.rows - r0);
    const int wrow0 = r0 + wave * kRowsPerWave;  // first row of this wave inside the task
    // Q' fragments (B operand): lane (ln, lg) holds 8 consecutive k of query row 16 i + ln
    Frag qf[QT][RK32];
#pragma unroll
    for (int i = 0; i < QT; ++i) {
      const int row = wrow0 + 16 * i + ln;
#pragma unroll
      for (int ks = 0; ks < RK32; ++ks) {
        const int col = 32 * ks + 8 * lg;
        qf[i][ks].u = (ks < rk32 && row < t.rows && col < rk)
                          ? *reinterpret_cast<const u32x4*>(q_lat + t.q_elem + (int64_t)row * t.ldq + col)
                          : u32x4{0, 0, 0, 0};
      }
    }
    f32x4 oacc[QT][RV16];
#pragma unroll
    for (int i = 0; i < QT; ++i)
#pragma unroll
      for (int c = 0; c < RV16; ++c) oacc[i][c] = f32x4{0.f, 0.f, 0.f, 0.f};
    // running maximum of the raw (unscaled) scores and running sum, per query row
    float m_run[QT], l_run[QT];
#pragma unroll
    for (int i = 0; i < QT; ++i) m_run[i] = -INFINITY, l_run[i] = 0.f;
    const int pos_base = t.pos0 + wrow0 + ln;  // absolute position of this lane's row in tile 0 (+16 for tile 1)

    const int last_pos = t.pos0 + r0 + pass_rows - 1;
    const int kv_end = causal ? min(t.kv_len, last_pos + 1) : t.kv_len;
    const bool wave_on = wrow0 < t.rows;
    const int wave_last_pos = t.pos0 + min(wrow0 + kRowsPerWave, t.rows) - 1;

    // register staging of the next block
    u32x4 kst[kSweeps], vst[kSweeps];   // E2M1: the chunk is the lower half
    auto fetch = [&](int c0) {  // rows past kv_len and lanes without a row read zeros through the range check
      __amdgpu_buffer_rsrc_t kr = k_rsrc, vr = v_rsrc;
      int rel = c0;
      if (t.page_tokens > 0) {
        // paged cache: the block lies inside one page (pages hold whole blocks); its rows are that
        // page's rows [rel, ..) of this head, valid up to the end of the page or of the sequence
        const int pi = c0 / t.page_tokens, start = pi * t.page_tokens;
        const int64_t pg = page_table[t.page_first + pi];
        const int rows = min(t.page_tokens, t.kv_len - start);
        kr = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(kbase + pg * page_stride_k * BITS / 8), 0, rows * rk * BITS / 8, 0x00020000);
        vr = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(vbase + pg * page_stride_v * BITS / 8), 0, rows * rv * BITS / 8, 0x00020000);
        rel = c0 - start;
      }
#pragma unroll
      for (int i = 0; i < kSweeps; ++i) {
        const int ko = (int)(k_goff[i] + (uint32_t)(rel * rk * BITS / 8)), vo = (int)(v_goff[i] + (uint32_t)(rel * rv * BITS / 8));
        if constexpr (kFp4) {
          if (i < k_sweeps) {
            const u32x2 c = __builtin_amdgcn_raw_buffer_load_b64(kr, ko, 0, 0);
            kst[i][0] = c[0], kst[i][1] = c[1];
          }
          if (i < v_sweeps) {
            const u32x2 c = __builtin_amdgcn_raw_buffer_load_b64(vr, vo, 0, 0);
            vst[i][0] = c[0], vst[i][1] = c[1];
          }
        } else {
          if (i < k_sweeps) kst[i] = __builtin_amdgcn_raw_buffer_load_b128(kr, ko, 0, 0);
          if (i < v_sweeps) vst[i] = __builtin_amdgcn_raw_buffer_load_b128(vr, vo, 0, 0);
        }
      }
    };
    auto put = [&](uint16_t* dst, const u32x4& chunk) {   // one 16-byte chunk of the cache -> bf16 in LDS
      if constexpr (BITS == 16) {
        *reinterpret_cast<u32x4*>(dst) = chunk;
      } else if constexpr (kFp4) {   // sixteen codes in two words -> sixteen bf16 (which holds every E2M1 value exactly),
        u32x4 lo, hi;                // two codes per instruction (v_cvt_scalef32_pk_bf16_fp4, scale 1; the byte select is an immediate)
#pragma unroll
        for (int w = 0; w < 2; ++w) {
          union { bf16x2 v; uint32_t u; } b0, b1, b2, b3;
          b0.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(chunk[w], 1.0f, 0);
          b1.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(chunk[w], 1.0f, 1);
          b2.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(chunk[w], 1.0f, 2);
          b3.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(chunk[w], 1.0f, 3);
          (w == 0 ? lo : hi) = u32x4{b0.u, b1.u, b2.u, b3.u};
        }
        *reinterpret_cast<u32x4*>(dst) = lo;
        *reinterpret_cast<u32x4*>(dst + 8) = hi;
      } else {   // sixteen E4M3 codes -> sixteen bf16, two per instruction (v_cvt_scalef32_pk_bf16_fp8, scale 1)
        u32x4 lo, hi;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          union { bf16x2 v; uint32_t u; } a, b;
          a.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(chunk[w], 1.0f, false);  // bytes 0, 1 of the word
          b.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(chunk[w], 1.0f, true);   // bytes 2, 3
          if (w < 2) lo[2 * w] = a.u, lo[2 * w + 1] = b.u;
          else hi[2 * (w - 2)] = a.u, hi[2 * (w - 2) + 1] = b.u;
        }
        *reinterpret_cast<u32x4*>(dst) = lo;
        *reinterpret_cast<u32x4*>(dst + 8) = hi;
      }
    };
    auto stage = [&](int buf) {
      uint16_t* lk = lds + buf * kStageElems;
      uint16_t* lv = lk + BCB * KROW;
#pragma unroll
      for (int i = 0; i < kSweeps; ++i) {
        if (i < k_sweeps && k_on[i]) put(&lk[k_loff[i]], kst[i]);
        if (i < v_sweeps && v_on[i]) put(&lv[v_loff[i]], vst[i]);
      }
    };

    __syncthreads();  // the previous pass / task (and the padding zeroing) is done with both buffers
    if (kv_end > 0) {
      fetch(0);
      stage(0);
      if (BCB < kv_end) fetch(BCB);
    }
    __syncthreads();
    int buf = 0;
    for (int cb = 0; cb < kv_end; cb += BCB, buf ^= 1) {
      const bool more = cb + BCB < kv_end;   // its rows are in flight or already in the staging registers
#pragma unroll
      for (int hf = 0; hf < NH; ++hf) {
      const int c0 = cb + hf * BC;
      if (c0 < kv_end && wave_on && !(causal && c0 > wave_last_pos)) {  // otherwise nothing visible for this wave (uniform)
        const uint16_t* lk = lds + buf * kStageElems + hf * BC * KROW;
        const uint16_t* lv = lds + buf * kStageElems + BCB * KROW + hf * BC * VROW;
        // S^T tiles: st[j][i] = tokens 16 j .. of the block x query rows of tile i
        f32x4 st[4][QT];
        score_tiles<RK32, QT>(lk, qf, st, ln, lg);
        // mask, online softmax. Lane (ln, lg) holds tokens c0 + 16 j + 4 lg + e of row ln.
        // p = 2^((s - m) * scale * log2 e) as one fma per score.
        const bool need_mask = (causal && c0 + BC - 1 > t.pos0 + wrow0) || c0 + BC > t.kv_len;
        Frag pf[QT][2];
#pragma unroll
        for (int i = 0; i < QT; ++i) {
          const int pos = pos_base + 16 * i;
          if (need_mask) {
            // only the sets on the causal diagonal and at the end of the keys come here; the empty statement keeps
            // the compiler from turning the branch into sixteen compares and selects that every set would execute
            asm volatile("" ::: "memory");
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const int tok = c0 + 16 * j + 4 * lg + e;
                if ((causal && tok > pos) || tok >= t.kv_len) st[j][i][e] = -INFINITY;
              }
          }
          float mx = -INFINITY;
#pragma unroll
          for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) mx = fmaxf(mx, st[j][i][e]);
          // The reference m of a row is raised only when the block beats it by kRaise (in log2 units of
          // the scaled score), so p stays below 2^kRaise and most blocks need no rescale of O at all.
          // The test needs no row maximum: a row beats its reference iff one of its four lanes does.
          if (__any(mx * scale_log2 > m_run[i] * scale_log2 + kRaise)) {
            mx = row_max(mx);
            const float m_new = fmaxf(m_run[i], mx);
            // a row with nothing visible yet keeps m = -inf; exp2(-inf - 0) = 0 scales the empty state
            const float m_ref = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f((m_run[i] - m_ref) * scale_log2);
            m_run[i] = m_new;
            l_run[i] *= alpha;
#pragma unroll
            for (int c = 0; c < RV16; ++c)
              if (c < rv16) oacc[i][c] *= alpha;
          }
          const float neg = m_run[i] == -INFINITY ? 0.f : -m_run[i] * scale_log2;
          float psum = 0.f;
          float p[4][4];
#pragma unroll
          for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              p[j][e] = __builtin_amdgcn_exp2f(fmaf(st[j][i][e], scale_log2, neg));
              psum += p[j][e];
            }
          l_run[i] += psum;
          // P^T operand of token pair-tiles (2 jp, 2 jp + 1): 8 bf16 per lane
#pragma unroll
          for (int jp = 0; jp < 2; ++jp) {
            pf[i][jp].u[0] = pack_bf16(p[2 * jp][0], p[2 * jp][1]);
            pf[i][jp].u[1] = pack_bf16(p[2 * jp][2], p[2 * jp][3]);
            pf[i][jp].u[2] = pack_bf16(p[2 * jp + 1][0], p[2 * jp + 1][1]);
            pf[i][jp].u[3] = pack_bf16(p[2 * jp + 1][2], p[2 * jp + 1][3]);
          }
        }
        pv_tiles<RV16, QT>(lv, pf, oacc, ln, lg);
      }
      }
      if (more) stage(buf ^ 1);  // the other buffer was last read before the previous barrier
      if (cb + 2 * BCB < kv_end) fetch(cb + 2 * BCB);   // requested before the barrier: its wait is part of the lead
      __syncthreads();
    }

    // finish: l over the four lanes of a row, normalise, store. Lane (ln, lg) holds O[row ln][16 c + 4 lg + e].
#pragma unroll
    for (int i = 0; i < QT; ++i) {
      const float l = row_sum(l_run[i]);
      const float inv = l > 0.f ? 1.f / l : 0.f;
      const int row = wrow0 + 16 * i + ln;
      if (row < t.rows) {
        uint16_t* orow = o_lat + t.o_elem + (int64_t)row * t.ldo;
#pragma unroll
        for (int c = 0; c < RV16; ++c) {
          if (c >= rv16) break;
          u32x2 w;
          w[0] = pack_bf16(oacc[i][c][0] * inv, oacc[i][c][1] * inv);
          w[1] = pack_bf16(oacc[i][c][2] * inv, oacc[i][c][3] * inv);
          *reinterpret_cast<u32x2*>(orow + 16 * c + 4 * lg) = w;
        }
      }
    }
  }
}

template <typename TC>
__global__ __launch_bounds__(kPreThreads) __attribute__((amdgpu_waves_per_eu(kPreWavesPerSimd, kPreWavesPerSimd))) void prefill_kernel(
    const PreTask* __restrict__ tasks, const int32_t* __restrict__ worker_ptr,
    const int32_t* __restrict__ worker_items, const uint16_t* __restrict__ q_lat,
    const TC* __restrict__ kc, const TC* __restrict__ vc, float scale_log2, int causal,
    uint16_t* __restrict__ o_lat, const int32_t* __restrict__ page_table, int64_t page_stride_k,
    int64_t page_stride_v) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[2 * kStageElems];
  const int w = blockIdx.x;
  const int i0 = worker_ptr[w], i1 = worker_ptr[w + 1];
  for (int it = i0; it < i1; ++it) {
    const PreTask t = tasks[worker_items[it]];
    // one copy of the task body per (k-steps, column tiles) class of the head; column-tile counts 5 and 7 round
    // up (the padded tile multiplies whatever the LDS columns behind a row's rank hold, stride padding or stale
    // data of a wider head, into accumulators of their own, and the output columns past rv are never stored)
    const int rk32 = ((t.rk_rv & 0xffff) + 31) / 32, rv16 = (t.rk_rv >> 16) / 16;
#define FDC_PRE(a, b) prefill_task<TC, a, b>(t, q_lat, kc, vc, scale_log2, causal, o_lat, page_table, page_stride_k, page_stride_v, lds)
#define FDC_PRE_ROW(a)                                      \
  switch (rv16) {                                           \
    case 1: FDC_PRE(a, 1); break;                           \
    case 2: FDC_PRE(a, 2); break;                           \
    case 3: FDC_PRE(a, 3); break;                           \
    case 4: FDC_PRE(a, 4); break;                           \
    case 5: case 6: FDC_PRE(a, 6); break;                   \
    default: FDC_PRE(a, 8); break;                          \
  }
    switch (rk32) {
      case 1: FDC_PRE_ROW(1) break;
      case 2: FDC_PRE_ROW(2) break;
      case 3: FDC_PRE_ROW(3) break;
      default: FDC_PRE_ROW(4) break;
    }
#undef FDC_PRE_ROW
#undef FDC_PRE
  }
}

fdc_status prefill_blocks_per_cu(int* nb) {
  FDC_HIP_CHECK(hipOccupancyMaxActiveBlocksPerMultiprocessor(nb, prefill_kernel<uint16_t>, kPreThreads, 0));
  return FDC_OK;
}

}  // namespace fdc

using namespace fdc;

extern "C" {

fdc_status fdc_latent_attn_prefill(const fdc_layout* lay, const fdc_plan* plan, const void* q_lat, const void* k_cache,
                                   const void* v_cache, float scale, int causal, void* o_lat, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  if (!lay || !plan || !q_lat || !k_cache || !v_cache || !o_lat || !workspace)
    FDC_FAIL(FDC_INVALID_ARG, "fdc_latent_attn_prefill: NULL argument");
  if (plan->kind != 1 || plan->lay != lay) FDC_FAIL(FDC_INVALID_ARG, "fdc_latent_attn_prefill: not a prefill plan of this layout");
  if (lay->dtype == FDC_F32) FDC_FAIL(FDC_UNSUPPORTED_DTYPE, "fdc_latent_attn_prefill: bf16 and E4M3 layouts only");
  if (!(scale > 0.f) || !(scale < 1e30f))
    FDC_FAIL(FDC_INVALID_ARG, "fdc_latent_attn_prefill: scale must be positive and finite (the running softmax orders scores by scale * s)");
  if (workspace_bytes < plan->workspace_bytes)
    FDC_FAIL(FDC_WORKSPACE_TOO_SMALL, "fdc_latent_attn_prefill: workspace has %zu bytes, the plan needs %zu",
             workspace_bytes, plan->workspace_bytes);
  if (!aligned16(q_lat) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(o_lat) ||
      (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
    FDC_FAIL(FDC_BAD_ALIGNMENT, "fdc_latent_attn_prefill: pointers must be 16-byte aligned (workspace 256)");
  if (plan->item_b.empty()) return FDC_OK;
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  auto go = [&](auto kern, auto* kp, auto* vp) {
    hipLaunchKernelGGL(kern, dim3(plan->n_workers), dim3(kPreThreads), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<const PreTask*>(ws + plan->off_items),
                       reinterpret_cast<const int32_t*>(ws + plan->off_worker_ptr),
                       reinterpret_cast<const int32_t*>(ws + plan->off_worker_items),
                       static_cast<const uint16_t*>(q_lat), kp, vp, scale * kLog2eP, causal,
                       static_cast<uint16_t*>(o_lat), reinterpret_cast<const int32_t*>(ws + plan->off_pages),
                       (int64_t)lay->max_seq * plan->RK, (int64_t)lay->max_seq * plan->RV);
  };
  if (lay->dtype == FDC_FP8)
    go(prefill_kernel<uint8_t>, static_cast<const uint8_t*>(k_cache), static_cast<const uint8_t*>(v_cache));
  else if (lay->dtype == FDC_FP4)
    go(prefill_kernel<fp4_t>, static_cast<const fp4_t*>(k_cache), static_cast<const fp4_t*>(v_cache));
  else
    go(prefill_kernel<uint16_t>, static_cast<const uint16_t*>(k_cache), static_cast<const uint16_t*>(v_cache));
  FDC_HIP_CHECK(hipGetLastError());
  return FDC_OK;
}

}  // extern "C"
