// Decode attention over the tiered KV cache, with cumulative-score emission (Eq. 1, Eq. 2-3 of the paper).
//
//   attn_tiered : grid (S, Hkv, B), one workgroup per compute unit.  The per-sequence lists F (T0 u T1 rows at full
//                 precision, ascending position) and Q (T2 rows, int8 / int4 codes) are cut into tiles of 64 entries;
//                 T3 positions are in neither list.  The S * NW waves of a (sequence, kv head) pair are divided
//                 between the two lists so that the longest wave is shortest, and every wave walks its tiles with a stride,
//                 on its own, with no workgroup barrier until the end.
//                 Rows never pass through registers on their way in: every lane fetches 16-byte (4-byte for short
//                 code rows) pieces straight into the wave's LDS tile buffer (buffer_load ... lds).  The one buffer
//                 holds the K rows of a tile, then its V rows, then the next tile's K rows: as soon as a piece has
//                 been read, the bytes it occupied are refilled with the pieces due next, so a wave keeps about a
//                 tile's worth of rows in flight while it computes; waits are vmcnt counts derived from the fixed
//                 issue order of one tile period.
//                   K rows  - 8 lanes per row; the G logits of a row are reduced over its 8 lanes by DPP and kept
//                             by the lane whose index equals the entry's index in the tile;
//                   softmax - online, one entry per lane (exact tile maximum, exp2, running m and l);
//                   V rows  - D/EV lanes per row, probabilities broadcast from LDS, per-lane fp32 output slices.
//                 The waves of a workgroup are merged through LDS into one split partial (m, l, o[G][D]); the scaled
//                 logits go to a scratch array.
//   attn_finish : grid (64-entry tiles + Hq, B).  Every workgroup first merges the (m, l) of all splits of its sequence
//                 into the global (m, 1/l) of every query head.  Tile workgroups then turn the stored logits
//                 into softmax weights, summed over all query heads in a fixed order, into score[b, pos]; the
//                 Hq remaining workgroups merge the split outputs of one query head each into out[b, hq].
//   attn_tiered_mc : the same launch for a chunk of query tokens (tkv_attend_and_score_chunk, 16-bit rows).  The
//                 tokens ride as extra columns beside the G heads of the group (up to 32 columns per workgroup), so
//                 a tile is fetched once for all of them: per tile a (64 rows x D) by (D x columns) product and its
//                 transpose-side twin for the output, which is a dense contraction and runs on the matrix cores
//                 (16x16x32 instructions; code rows widened to 16-bit values in LDS first).  attn_finish_chunk
//                 adds the tokens' weights to the scores in token order.
// The tile boundaries, the wave assignment and the fp32 summation order depend only on the lists' logical order and
// lengths, never on whether a row lives in the HBM pool or the staging buffer (both are one slot space), which is
// what makes T1 placement bit-invisible (Prop. 1).  A decode step (one query token) uses no matrix instructions: the
// launch is bound by HBM, and the per-row work is G dot products.
#include <hip/hip_ext.h>

#include <utility>

#include "tkv_internal.h"

namespace tkv {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(3))) char lds_char;

constexpr float LOG2E = 1.4426950408889634f;
constexpr int TB = TOK_PER_BLOCK;
static_assert(TB == 64, "a tile is one list entry per lane");

enum Mode : int { F_BF16 = 0, F_F32 = 1, Q_INT8 = 2, Q_INT4 = 3, F_F16 = 4 };
// type of K, V and q as a template argument: binary32, bfloat16, binary16
constexpr int KT_F32 = 0, KT_BF16 = 1, KT_F16 = 2;

template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): loop indices usable as immediates
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// at most N vector-memory operations of this wave still outstanding (they complete in issue order)
template <int N>
__device__ __forceinline__ void wait_vm() {
  constexpr int n = N > 63 ? 63 : (N < 0 ? 0 : N);
  __builtin_amdgcn_s_waitcnt((n & 15) | ((n >> 4) << 14) | 0x0F70);
}

// ---- LDS accesses the compiler's wait insertion does not see ------------------------------------------------
// A compiler-visible LDS load issued while direct-to-LDS loads are outstanding is preceded by a wait for all of
// them, which would serialise the pipeline; the waits for these are placed by hand (lds_fence).
template <int OFF>
__device__ __forceinline__ u32x4 lds_rd128(uint32_t addr) {
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
template <int OFF>
__device__ __forceinline__ u32x2 lds_rd64(uint32_t addr) {
  u32x2 v;
  asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}
template <int OFF>
__device__ __forceinline__ uint32_t lds_rd32(uint32_t addr) {
  uint32_t v;
  asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}
// Transposing read: within every 16 lanes, the 4 lanes 4j .. 4j+3 point at 4 x 8 bytes that together are 16
// consecutive 16-bit elements of matrix row j (j < 4); lane i of the 16 receives element i of rows 0..3.
template <int OFF>
__device__ __forceinline__ u32x2 lds_rd64_tr16(uint32_t addr) {
  u32x2 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}
template <int OFF>
__device__ __forceinline__ void lds_wr128(uint32_t addr, u32x4 v) {
  asm volatile("ds_write_b128 %0, %1 offset:%2" : : "v"(addr), "v"(v), "n"(OFF) : "memory");
}
__device__ __forceinline__ void lds_wr32(uint32_t addr, uint32_t v) {
  asm volatile("ds_write_b32 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_wait() { asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory"); }
// values read by lds_rd* may be used only after lds_wait() and tie() of the variable
__device__ __forceinline__ void tie(u32x4& v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void tie(uint32_t& v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void tie(u32x2& v) { asm volatile("" : "+v"(v)); }
template <class T, int N>
__device__ __forceinline__ void tie(T (&v)[N]) {
#pragma unroll
  for (int i = 0; i < N; ++i) tie(v[i]);
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(size_t)(const lds_char*)p;
}

template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
  return __builtin_amdgcn_update_dpp(0.f, x, CTRL, 0xf, 0xf, false);
}
// rows listed in ROW_MASK receive the DPP source, the others keep x
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_rows(float x) {
  return __builtin_amdgcn_update_dpp(x, x, CTRL, ROW_MASK, 0xf, false);
}

// sum over aligned groups of LPR consecutive lanes; every lane of the group receives the result
template <int LPR>
__device__ __forceinline__ float group_sum(float x) {
  if constexpr (LPR >= 2) x += dpp_f<0xB1>(x);    // quad_perm [1,0,3,2]
  if constexpr (LPR >= 4) x += dpp_f<0x4E>(x);    // quad_perm [2,3,0,1]
  if constexpr (LPR >= 8) x += dpp_f<0x141>(x);   // row_half_mirror
  if constexpr (LPR >= 16) x += dpp_f<0x140>(x);  // row_mirror
  return x;
}
__device__ __forceinline__ float rdlane(float x, int l) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), l));
}

// whole-wave reductions: 16-lane rows by DPP, rows 0/1 and 2/3 by row_bcast15, halves by row_bcast31; lane 63 has
// the result, which is returned in a scalar register
// Whole-wave maxima of G values at once: 16-lane rows by DPP (quad swaps, half mirror, mirror), then row_bcast15
// (lane 15 of a row into the next row) and row_bcast31 (lane 31 into the upper half); afterwards LANE 63 ALONE holds
// the maximum of each value (the other lanes are not kept consistent by the last two steps).  The DPP form of v_max
// is written out because the compiler would put a quieting v_max and a separate DPP move around every step.  A DPP
// operand may not be read in the two instructions after the one that wrote it: the steps go value by value, so with
// three or more values the other values' instructions fill that gap, otherwise an s_nop does.  The values may come
// straight out of dot instructions, whose results an ordinary VALU instruction may not read for three instructions
// (the compiler pads its own code for this, not inline asm): hence the longer s_nop before the first step.  Source
// and destination are separate operands, so the register allocator has no reason to slip a copy in front of a step.
template <int G>
__device__ __forceinline__ void wave_max_all(float (&x)[G]) {
#define TKV_MAX_STEP(CTRL)                                                                             \
  _Pragma("unroll") for (int h = 0; h < G; ++h) {                                                      \
    float r;                                                                                           \
    if (G < 3 || h == 0) asm volatile("s_nop 1");                                                      \
    asm volatile("v_max_f32_dpp %0, %1, %1 " CTRL : "=v"(r) : "v"(x[h]));                              \
    x[h] = r;                                                                                          \
  }
  // every value is in its register before the first step, and its writer is far enough behind
  _Pragma("unroll") for (int h = 0; h < G; ++h) asm volatile("" : : "v"(x[h]));
  asm volatile("s_nop 3");
  TKV_MAX_STEP("quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf")
  TKV_MAX_STEP("quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf")
  TKV_MAX_STEP("row_half_mirror row_mask:0xf bank_mask:0xf")
  TKV_MAX_STEP("row_mirror row_mask:0xf bank_mask:0xf")
  TKV_MAX_STEP("row_bcast:15 row_mask:0xa bank_mask:0xf")
  TKV_MAX_STEP("row_bcast:31 row_mask:0xc bank_mask:0xf")
#undef TKV_MAX_STEP
}
// Sums of G values over aligned groups of 8 lanes, every lane of a group receiving the result; same scheme (and the
// same reason for writing the DPP form out) as wave_max_all.
template <int G>
__device__ __forceinline__ void group_sum8_all(float (&x)[G]) {
#define TKV_ADD_STEP(CTRL)                                                                             \
  _Pragma("unroll") for (int h = 0; h < G; ++h) {                                                      \
    float r;                                                                                           \
    if (G < 3 || h == 0) asm volatile("s_nop 1");                                                      \
    asm volatile("v_add_f32_dpp %0, %1, %1 " CTRL : "=v"(r) : "v"(x[h]));                              \
    x[h] = r;                                                                                          \
  }
  _Pragma("unroll") for (int h = 0; h < G; ++h) asm volatile("" : : "v"(x[h]));
  asm volatile("s_nop 3");
  TKV_ADD_STEP("quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf")
  TKV_ADD_STEP("quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf")
  TKV_ADD_STEP("row_half_mirror row_mask:0xf bank_mask:0xf")
#undef TKV_ADD_STEP
}
__device__ __forceinline__ float wave_sum(float x) {
  x = group_sum<16>(x);
  const float a = rdlane(x, 0) + rdlane(x, 16), b = rdlane(x, 32) + rdlane(x, 48);
  return a + b;
}

__device__ __forceinline__ float bf_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __builtin_bit_cast(float, u & 0xffff0000u); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
// two code values (exact in binary16) packed as a binary16 pair
__device__ __forceinline__ uint32_t pack_f16_pair(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}
__device__ __forceinline__ float f16_lo(uint32_t u) { return (float)__builtin_bit_cast(f16x2, u).x; }
__device__ __forceinline__ float f16_hi(uint32_t u) { return (float)__builtin_bit_cast(f16x2, u).y; }
// two code values (exact in bf16: at most 8 significant bits) packed as a bf16 pair
__device__ __forceinline__ uint32_t pack_bf16_pair(float lo, float hi) {
  return (__builtin_bit_cast(uint32_t, hi) & 0xffff0000u) | (__builtin_bit_cast(uint32_t, lo) >> 16);
}
__device__ __forceinline__ float half_of(uint32_t w, int hi) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)(hi ? (w >> 16) : (w & 0xffffu)));
}

template <int G>
struct GPad { static constexpr int v = (G <= 4) ? 4 : 8; };

// ---- geometry ------------------------------------------------------------------------------------------------
// A row is fetched in "units" of 16 bytes (4 bytes where a lane's share of a row is shorter than 16), one unit per
// lane and direct-to-LDS instruction; the lane that fetched a unit is the lane that reads it back.
//   K side: 8 lanes per row; lane r8 owns units j*8 + r8, j < KU          (K batch i = rows 8*g8 + i, g8 = lane/8)
//   V side: LPRV lanes per row; lane rv owns units rv*VU + u, u < VU      (V step it = rows LPRV*gv + it, gv = lane/LPRV)
template <int D, Mode M>
struct Geo {
  static constexpr bool IS_Q = (M == Q_INT8 || M == Q_INT4);
  static constexpr int RB = (M == F_BF16 || M == F_F16) ? 2 * D : (M == F_F32) ? 4 * D : (M == Q_INT8) ? D : D / 2;   // bytes per row
  static constexpr int KLB = RB / 8;                        // bytes of a K row per lane
  static constexpr int KS = (KLB % 16 == 0) ? 16 : 4;       // bytes per unit
  static constexpr int KU = KLB / KS;                       // units per lane and row
  static constexpr int EUK = KS * D / RB;                   // elements per unit
  static constexpr int EV = (M == F_F32) ? 4 : 8;           // elements of a V row per lane
  static constexpr int LPRV = D / EV;                       // lanes per V row
  static constexpr int NITV = LPRV;                         // V steps per tile
  static constexpr int VLB = RB / LPRV;                     // bytes of a V row per lane
  static constexpr int VS = (VLB % 16 == 0) ? 16 : 4;
  static constexpr int VU = VLB / VS;
  static constexpr int EUV = EV / VU;                       // elements per V unit
  static constexpr int SCD = (M == Q_INT8) ? 1 : (M == Q_INT4) ? D / 64 : 0;   // dwords of scales per row
  static constexpr float OFF = (M == Q_INT4) ? 8.f : 128.f; // codes are read as code + OFF
  // direct-to-LDS operations of one tile period, in issue order: slot list, K scales, K batches, V scales, V steps
  static constexpr int N_K = 8 * KU, N_V = NITV * VU;
  static constexpr int T = 1 + SCD + N_K + SCD + N_V;
  static_assert(KLB % KS == 0 && VLB % VS == 0 && LPRV % 4 == 0 && (!IS_Q || D % 64 == 0), "unsupported head_dim");
};

template <int S>
struct UnitT { using type = uint32_t; };
template <>
struct UnitT<16> { using type = u32x4; };

// element c of a vector, by value (a bit cast applied directly to a vector element reads element 0)
__device__ __forceinline__ uint32_t elem(const u32x4& v, int c) { return v[c]; }
__device__ __forceinline__ float elem_f(const u32x4& v, int c) { const uint32_t w = v[c]; return __builtin_bit_cast(float, w); }

template <int S>
__device__ __forceinline__ uint32_t unit_word(const typename UnitT<S>::type& u, int c) {
  if constexpr (S == 16) return u[c]; else return u;
}

// codes of one unit as unsigned values code + OFF; the offset is removed once per row (sum q*(u-OFF) = sum q*u - OFF*sum q)
template <Mode M, int S, int E>
__device__ __forceinline__ void unpack_unit(const typename UnitT<S>::type& u, float (&f)[E]) {
  if constexpr (M == Q_INT8) {
#pragma unroll
    for (int i = 0; i < S / 4; ++i) {
      const uint32_t w = unit_word<S>(u, i) ^ 0x80808080u;
#pragma unroll
      for (int n = 0; n < 4; ++n) f[i * 4 + n] = (float)((w >> (8 * n)) & 0xFFu);
    }
  } else {
#pragma unroll
    for (int i = 0; i < S / 4; ++i) {
      const uint32_t w = unit_word<S>(u, i) ^ 0x88888888u;
#pragma unroll
      for (int n = 0; n < 8; ++n) f[i * 8 + n] = (float)((w >> (4 * n)) & 0xFu);
    }
  }
}

// The lane's units of the G query vectors.  bf16 queries stay packed (fed to the bf16 dot instruction); binary32
// queries are kept as floats.  qs is the sum over a unit (Q modes only).
template <int D, int G, Mode M, int KT>
struct QRegs {
  using GE = Geo<D, M>;
  static constexpr bool QBF = KT != KT_F32;   // 16-bit queries stay packed in pairs
  uint32_t qp[QBF ? G : 1][GE::KU][GE::EUK / 2];
  float qf[QBF ? 1 : G][GE::KU][GE::EUK];
  float qs[G][GE::KU];
};

template <int D, Mode M>
struct KBatch { typename UnitT<Geo<D, M>::KS>::type u[Geo<D, M>::KU]; };
template <int D, int G, Mode M>
struct VStep {
  typename UnitT<Geo<D, M>::VS>::type u[Geo<D, M>::VU];
  u32x4 p[GPad<G>::v / 4];
};

// G logits of one K row, reduced over the row's 8 lanes (every lane of the group gets them).
// sc: INT8 the row's scale; INT4 the scale of the 32-code group of each of the lane's units.
template <int D, int G, Mode M, int KT>
__device__ __forceinline__ void row_logits(const KBatch<D, M>& kr, const QRegs<D, G, M, KT>& q,
                                           const float (&sc)[Geo<D, M>::KU], float (&x)[G]) {
  using GE = Geo<D, M>;
  constexpr int KU = GE::KU, KS = GE::KS, EUK = GE::EUK;
  constexpr bool QBF = KT != KT_F32, H = KT == KT_F16;
  if constexpr (M == F_F16) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float acc = 0.f;
#pragma unroll
      for (int j = 0; j < KU; ++j)
#pragma unroll
        for (int c = 0; c < EUK / 2; ++c)
          acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, unit_word<KS>(kr.u[j], c)),
                                       __builtin_bit_cast(f16x2, q.qp[h][j][c]), acc, false);
      x[h] = acc;
    }
    group_sum8_all<G>(x);
  } else if constexpr (M == F_BF16) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float acc = 0.f;
#pragma unroll
      for (int j = 0; j < KU; ++j)
#pragma unroll
        for (int c = 0; c < EUK / 2; ++c)
          acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, unit_word<KS>(kr.u[j], c)),
                                                __builtin_bit_cast(bf16x2, q.qp[h][j][c]), acc, false);
      x[h] = acc;
    }
    group_sum8_all<G>(x);
  } else if constexpr (M == F_F32) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float acc = 0.f;
#pragma unroll
      for (int j = 0; j < KU; ++j)
#pragma unroll
        for (int c = 0; c < EUK; ++c) acc = fmaf(__builtin_bit_cast(float, unit_word<KS>(kr.u[j], c)), q.qf[h][j][c], acc);
      x[h] = acc;
    }
    group_sum8_all<G>(x);
  } else {
    float tot[G];
#pragma unroll
    for (int h = 0; h < G; ++h) tot[h] = 0.f;
#pragma unroll
    for (int j = 0; j < KU; ++j) {
      float kf[EUK];
      unpack_unit<M, KS, EUK>(kr.u[j], kf);
      uint32_t kp[EUK / 2];
      if constexpr (QBF) {
#pragma unroll
        for (int c = 0; c < EUK / 2; ++c) kp[c] = H ? pack_f16_pair(kf[2 * c], kf[2 * c + 1]) : pack_bf16_pair(kf[2 * c], kf[2 * c + 1]);
      }
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float acc = -GE::OFF * q.qs[h][j];
        if constexpr (QBF) {
#pragma unroll
          for (int c = 0; c < EUK / 2; ++c) {
            if constexpr (H) acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, kp[c]), __builtin_bit_cast(f16x2, q.qp[h][j][c]), acc, false);
            else acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, kp[c]), __builtin_bit_cast(bf16x2, q.qp[h][j][c]), acc, false);
          }
        } else {
#pragma unroll
          for (int c = 0; c < EUK; ++c) acc = fmaf(q.qf[h][j][c], kf[c], acc);
        }
        if constexpr (M == Q_INT4) tot[h] = fmaf(acc, sc[j], tot[h]);   // per-group scale: before the cross-lane sum
        else tot[h] += acc;
      }
    }
    group_sum8_all<G>(tot);
#pragma unroll
    for (int h = 0; h < G; ++h) {
      x[h] = tot[h];
      if constexpr (M == Q_INT8) x[h] *= sc[0];                         // per-row scale
    }
  }
}

// o[h][e] += p[h] * v[e] for the lane's EV elements of one V row (Q modes: p scaled, offset handled through osub)
template <int D, int G, Mode M>
__device__ __forceinline__ void row_accumulate(const VStep<D, G, M>& vr, float sc, float (&o)[G][Geo<D, M>::EV], float (&osub)[G]) {
  using GE = Geo<D, M>;
  constexpr int EV = GE::EV, VU = GE::VU, VS = GE::VS, EUV = GE::EUV;
  float p[GPad<G>::v];
#pragma unroll
  for (int c = 0; c < GPad<G>::v; ++c) p[c] = elem_f(vr.p[c / 4], c % 4);
  float vf[EV];
  if constexpr (M == F_BF16) {
#pragma unroll
    for (int c = 0; c < 4; ++c) { const uint32_t wv = elem(vr.u[0], c); vf[2 * c] = bf_lo(wv); vf[2 * c + 1] = bf_hi(wv); }
  } else if constexpr (M == F_F16) {
#pragma unroll
    for (int c = 0; c < 4; ++c) { const uint32_t wv = elem(vr.u[0], c); vf[2 * c] = f16_lo(wv); vf[2 * c + 1] = f16_hi(wv); }
  } else if constexpr (M == F_F32) {
#pragma unroll
    for (int c = 0; c < 4; ++c) vf[c] = elem_f(vr.u[0], c);
  } else {
#pragma unroll
    for (int u = 0; u < VU; ++u) {
      float t[EUV];
      unpack_unit<M, VS, EUV>(vr.u[u], t);
#pragma unroll
      for (int e = 0; e < EUV; ++e) vf[u * EUV + e] = t[e];
    }
  }
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float ph = p[h];
    if constexpr (GE::IS_Q) { ph *= sc; osub[h] += ph; }
#pragma unroll
    for (int e = 0; e < EV; ++e) o[h][e] = fmaf(ph, vf[e], o[h][e]);
  }
}

// LDS regions of one wave (pointers for the direct loads, byte addresses for the reads)
struct WaveLds {
  char* t; char* sk; char* sv; char* lt;   // tile buffer (K rows, then V rows, in turn), K scales, V scales, slot lists (2 x 64 ints)
  char* p;                                 // probabilities of the current tile (before the first tile: the query block)
  uint32_t ta, ska, sva, lta, pa;          // the same as LDS addresses
};

template <int SZ>
__device__ __forceinline__ void dma(const __amdgpu_buffer_rsrc_t& rs, char* lds, uint32_t voff, int aux) {
  static_assert(SZ == 16 || SZ == 4, "unit sizes");
  if constexpr (SZ == 16) {
    if (aux) __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)lds, 16, voff, 0, 0, 2);
    else __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)lds, 16, voff, 0, 0, 0);
  } else {
    if (aux) __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)lds, 4, voff, 0, 0, 2);
    else __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)lds, 4, voff, 0, 0, 0);
  }
}

// ---- one wave: the tiles tile0, tile0 + tstride, ... of one list ------------------------------------------------
// One tile buffer per wave holds the K rows of a tile, then its V rows, then the next tile's K rows: a K batch that
// has been read is refilled with the V pieces that fall on the same bytes, a V step with K pieces of the next tile.
// Issue order of one tile period (the vmcnt arguments below are counts of younger operations in this order):
//   slot list of tile t+2 | K scales of t+1 | per K batch of t: the V pieces of t on its bytes |
//   V scales of t+1 | per V step of t: the K pieces of t+1 on its bytes
// Accumulates into o (offset-corrected for code rows), m_run, l_lane (per-lane partial sums of the softmax
// denominator, relative to m_run); leaves the scaled logits in xs.
template <int D, int G, Mode M, int KT>
__device__ __forceinline__ void attn_wave(const AttnArgs& a, const WaveLds& w, int b, int jq, int kvh, int lane,
                                          int tile0, int tstride, int n_list, const int* loc_list, int xs_tile0,
                                          float (&o)[G][Geo<D, M>::EV], float (&m_run)[G], float (&l_lane)[G]) {
  using GE = Geo<D, M>;
  constexpr int EV = GE::EV, LPRV = GE::LPRV, NITV = GE::NITV, KU = GE::KU, KS = GE::KS, VU = GE::VU, VS = GE::VS;
  constexpr int EUK = GE::EUK, SCD = GE::SCD, RB = GE::RB, N_K = GE::N_K, N_V = GE::N_V;
  constexpr int GP = GPad<G>::v;
  constexpr bool QBF = KT != KT_F32, H = KT == KT_F16;
  constexpr int KIB = 64 * KS, VIB = 64 * VS;        // bytes of the tile buffer one K / V piece covers
  constexpr int KBB = KU * KIB, VSB = VU * VIB;      // ... one K batch / one V step
  static_assert(KBB % VIB == 0 && 8 * KBB == NITV * VSB, "K batches and V steps tile the same buffer");
  constexpr int VPB = KBB / VIB;                     // V pieces issued after each K batch
  const int g8 = lane >> 3, r8 = lane & 7;           // K side: row group and unit column
  const int gv = lane / LPRV, rv = lane % LPRV;      // V side

  __amdgpu_buffer_rsrc_t rk, rvv, rsk, rsv;
  if constexpr (!GE::IS_Q) {
    const size_t off = (size_t)(b * a.Hkv + kvh) * a.capF * RB;
    rk = make_rsrc(a.fpK + off, (uint32_t)a.capF * RB); rvv = make_rsrc(a.fpV + off, (uint32_t)a.capF * RB);
    rsk = rk; rsv = rvv;
  } else {
    const size_t rows = (size_t)(b * a.Hkv + kvh) * a.cap2;
    rk = make_rsrc(a.c2K + rows * a.cb, (uint32_t)a.cap2 * a.cb); rvv = make_rsrc(a.c2V + rows * a.cb, (uint32_t)a.cap2 * a.cb);
    rsk = make_rsrc(a.s2K + rows * a.sb, (uint32_t)a.cap2 * a.sb); rsv = make_rsrc(a.s2V + rows * a.sb, (uint32_t)a.cap2 * a.sb);
  }
  const __amdgpu_buffer_rsrc_t rl = make_rsrc(loc_list, (uint32_t)a.Nmax * 4u);

  if (tile0 * 64 >= n_list) return;

  // The first tile's slot list is asked for before anything else: the compute unit serves its waves' requests in
  // the order they were made, and a list request that came behind another wave's rows would wait for all of them.
  dma<4>(rl, w.lt, (uint32_t)(tile0 * 64 + lane) * 4u, 0);

  // The lane's units of the G query vectors.  16-bit queries (G * D * 2 bytes, contiguous) come in through the
  // probability region of the LDS, as NQD direct loads of 1 KB whose count the waits below can name; binary32
  // queries are fetched by ordinary loads (the wait for the list then waits for them as well).
  QRegs<D, G, M, KT> q;
  constexpr int NQD = QBF ? (G * D * 2 + 1023) / 1024 : 0;
  static_assert(NQD * 1024 <= 64 * GP * 4, "the query block is parked in the probability region");
  if constexpr (QBF) {
    const char* qb = (const char*)a.q + ((size_t)b * a.q_bs + (size_t)jq * a.Hq + kvh * G) * D * 2;
    const __amdgpu_buffer_rsrc_t rq = make_rsrc(qb, (uint32_t)(G * D * 2));   // lanes past the block fetch zeros
#pragma unroll
    for (int i = 0; i < NQD; ++i) dma<16>(rq, w.p + i * 1024, (uint32_t)(i * 1024 + lane * 16), 0);
  } else {
    const char* qb = (const char*)a.q + ((size_t)b * a.q_bs + (size_t)jq * a.Hq + kvh * G) * D * 4;
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int j = 0; j < KU; ++j) {
        const char* src = qb + ((size_t)h * D + (size_t)(j * 8 + r8) * EUK) * 4;
        float sacc = 0.f;
#pragma unroll
        for (int c = 0; c < EUK; ++c) {
          q.qf[h][j][c] = ((const float*)src)[c];
          if constexpr (GE::IS_Q) sacc += q.qf[h][j][c];
        }
        q.qs[h][j] = sacc;
      }
  }

  float osub[G];
#pragma unroll
  for (int h = 0; h < G; ++h) osub[h] = 0.f;

  // per-lane byte offsets of its units within a row, and its LDS read addresses
  const uint32_t kcol = (uint32_t)r8 * KS, vcol = (uint32_t)rv * (VU * VS);
  const uint32_t k_rd = w.ta + (uint32_t)lane * KS, v_rd = w.ta + (uint32_t)lane * VS;
  const uint32_t p_wr = w.pa + (uint32_t)lane * (GP * 4), p_rd = w.pa + (uint32_t)(gv * LPRV) * (GP * 4);

  // slots of the rows this lane fetches: lk / lrow belong to the tile whose K rows are fetched next, lv to the
  // tile whose V rows are fetched next
  int lk[8], lv[LPRV], lrow;
  // reads the K-side slots (rows 8*g8 + i) and the lane's own row's slot of the list in LDS half `par`
  auto read_locs_k = [&](int par, int nvalid) {
    const uint32_t base = w.lta + (uint32_t)par * 256u;
    if (nvalid < 64) {                                   // wave-uniform: a list's last tile
      if (lane >= nvalid) lds_wr32(base + (uint32_t)lane * 4u, 0xffffffffu);   // no row: fetches land as zeros
    }
    u32x4 t0 = lds_rd128<0>(base + (uint32_t)g8 * 32u), t1 = lds_rd128<16>(base + (uint32_t)g8 * 32u);
    uint32_t me = lds_rd32<0>(base + (uint32_t)lane * 4u);
    lds_wait(); tie(t0); tie(t1); tie(me);
    lk[0] = t0.x; lk[1] = t0.y; lk[2] = t0.z; lk[3] = t0.w; lk[4] = t1.x; lk[5] = t1.y; lk[6] = t1.z; lk[7] = t1.w;
    lrow = (int)me;
  };
  auto read_locs_v = [&](int par) {
    const uint32_t base = w.lta + (uint32_t)par * 256u + (uint32_t)(gv * LPRV) * 4u;
    u32x4 t[LPRV / 4];
    static_for<LPRV / 4>([&](auto cc) { constexpr int c = decltype(cc)::value; t[c] = lds_rd128<c * 16>(base); });
    lds_wait(); tie(t);
#pragma unroll
    for (int c = 0; c < LPRV / 4; ++c) { lv[4 * c] = t[c].x; lv[4 * c + 1] = t[c].y; lv[4 * c + 2] = t[c].z; lv[4 * c + 3] = t[c].w; }
  };
  auto issue_loc = [&](int par, int tile) {
    dma<4>(rl, w.lt + par * 256, (uint32_t)(tile * 64 + lane) * 4u, 0);
  };
  auto issue_kscale = [&]() {
#pragma unroll
    for (int j = 0; j < SCD; ++j) dma<4>(rsk, w.sk + j * 256, (uint32_t)lrow * (uint32_t)a.sb + j * 4u, 0);
  };
  auto issue_vscale = [&]() {
#pragma unroll
    for (int j = 0; j < SCD; ++j) dma<4>(rsv, w.sv + j * 256, (uint32_t)lrow * (uint32_t)a.sb + j * 4u, 0);
  };
  auto issue_k_piece = [&](int s) {                      // K piece s = (batch s / KU, unit s % KU)
    const int i = s / KU, j = s % KU;
    dma<KS>(rk, w.t + s * KIB, (uint32_t)lk[i] * (uint32_t)RB + (uint32_t)j * (8 * KS) + kcol, 1);
  };
  auto issue_v_piece = [&](int v) {                      // V piece v = (step v / VU, unit v % VU)
    const int it = v / VU, u = v % VU;
    dma<VS>(rvv, w.t + v * VIB, (uint32_t)lv[it] * (uint32_t)RB + vcol + (uint32_t)u * VS, 1);
  };

  // ---- prologue: the first tile's slot list has been asked for; then its scales and K rows in the order of a tile
  // period, and the query block out of the LDS into registers
  wait_vm<NQD>();                                        // the list is in (binary32 queries: and the queries)
  read_locs_k(0, n_list - tile0 * 64);
  issue_loc(1, tile0 + tstride);
  issue_kscale();
  issue_vscale();
#pragma unroll
  for (int s = 0; s < N_K; ++s) issue_k_piece(s);
  if constexpr (QBF) {
    wait_vm<1 + 2 * SCD + N_K>();                        // everything older than the second list: the query block
    // a unit of a query is EUK 16-bit elements: 8 bytes (one ds_read_b64) or QB pieces of 16
    constexpr int QW = EUK / 2, QB = QW / 4;
    static_assert(QW == 2 || QW % 4 == 0, "query units are 8 bytes or whole 16-byte pieces");
    const uint32_t q_rd = w.pa + (uint32_t)r8 * (EUK * 2);
    if constexpr (QW == 2) {
      u32x2 t[G][KU];
      static_for<G>([&](auto hc) {
        constexpr int h = decltype(hc)::value;
        static_for<KU>([&](auto jc) { constexpr int j = decltype(jc)::value; t[h][j] = lds_rd64<h * D * 2 + j * 8 * EUK * 2>(q_rd); });
      });
      lds_wait();
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int j = 0; j < KU; ++j) { tie(t[h][j]); q.qp[h][j][0] = t[h][j].x; q.qp[h][j][1] = t[h][j].y; }
    } else {
      u32x4 t[G][KU][QB > 0 ? QB : 1];
      static_for<G>([&](auto hc) {
        constexpr int h = decltype(hc)::value;
        static_for<KU>([&](auto jc) {
          constexpr int j = decltype(jc)::value;
          static_for<QB>([&](auto cc) { constexpr int c = decltype(cc)::value; t[h][j][c] = lds_rd128<h * D * 2 + j * 8 * EUK * 2 + c * 16>(q_rd); });
        });
      });
      lds_wait();
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int j = 0; j < KU; ++j)
#pragma unroll
          for (int c = 0; c < QB; ++c) {
            tie(t[h][j][c]);
#pragma unroll
            for (int e = 0; e < 4; ++e) q.qp[h][j][c * 4 + e] = elem(t[h][j][c], e);
          }
    }
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int j = 0; j < KU; ++j) {
        float sacc = 0.f;
        if constexpr (GE::IS_Q) {
#pragma unroll
          for (int c = 0; c < QW; ++c) sacc += H ? f16_lo(q.qp[h][j][c]) + f16_hi(q.qp[h][j][c]) : bf_lo(q.qp[h][j][c]) + bf_hi(q.qp[h][j][c]);
        }
        q.qs[h][j] = sacc;
      }
  }

  int par = 1;                                           // LDS half that holds the next tile's slot list
  auto tile_body = [&](int tile, auto more_c) {
    constexpr bool MORE = decltype(more_c)::value;
    constexpr int X = MORE ? 1 : 0;                      // operations of the parts a last tile does not issue
    const bool valid = tile * 64 + lane < n_list;
    // The two waves of a SIMD are issued oldest first, which lets the first wave of a pair run a whole tile ahead and
    // leaves the second one to finish on its own; the wave with more phases still to do goes first instead.
    __builtin_amdgcn_s_setprio(MORE ? 3 : 1);
    // -- V-side slots of this tile; K-side slots of the next one; fetch the list after that
    read_locs_v(par ^ 1);
    if constexpr (MORE) {
      wait_vm<2 * SCD + N_K>();
      read_locs_k(par, n_list - (tile + tstride) * 64);
      issue_loc(par ^ 1, tile + 2 * tstride);
    }
    // -- K scales of this tile
    float ksc[8][KU];
    if constexpr (GE::IS_Q) {
      wait_vm<SCD + N_K + X>();
      u32x4 t[SCD][2];
      static_for<SCD>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        t[j][0] = lds_rd128<j * 256>(w.ska + (uint32_t)g8 * 32u);
        t[j][1] = lds_rd128<j * 256 + 16>(w.ska + (uint32_t)g8 * 32u);
      });
      lds_wait();
#pragma unroll
      for (int j = 0; j < SCD; ++j) { tie(t[j][0]); tie(t[j][1]); }
      if constexpr (MORE) issue_kscale();
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < KU; ++j) {
          if constexpr (M == Q_INT8) ksc[i][j] = elem_f(t[0][i / 4], i % 4);
          else ksc[i][j] = half_of(elem(t[j][i / 4], i % 4), (r8 >> 2) & 1);   // unit j*8 + r8 lies in group 2*j + r8/4
        }
    }
    // -- K rows: read batch i+1 while batch i is computed; a batch that has been read is refilled with V pieces
    float xt[G];
#pragma unroll
    for (int h = 0; h < G; ++h) xt[h] = 0.f;
    KBatch<D, M> kb[2];
    auto read_k = [&](auto ic, KBatch<D, M>& dst) {
      constexpr int i = decltype(ic)::value;
      // younger than this batch's pieces: the later K pieces, the list and K-scale fetches of this period, the V pieces so far
      wait_vm<N_K - 1 - ((i + 1) * KU - 1) + X * (1 + SCD) + i * VPB>();
      static_for<KU>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        if constexpr (KS == 16) dst.u[j] = lds_rd128<(i * KU + j) * KIB>(k_rd);
        else dst.u[j] = lds_rd32<(i * KU + j) * KIB>(k_rd);
      });
    };
    read_k(std::integral_constant<int, 0>{}, kb[0]);
    static_for<8>([&](auto ic) {
      constexpr int i = decltype(ic)::value;
      lds_wait(); tie(kb[i & 1].u);
#pragma unroll
      for (int v = i * VPB; v < (i + 1) * VPB; ++v) issue_v_piece(v);
      if constexpr (i + 1 < 8) read_k(std::integral_constant<int, (i + 1 < 8 ? i + 1 : 7)>{}, kb[(i + 1) & 1]);
      float x[G];
      row_logits<D, G, M, KT>(kb[i & 1], q, ksc[i], x);
#pragma unroll
      for (int h = 0; h < G; ++h) xt[h] = (r8 == i) ? x[h] : xt[h];   // lane 8*g8 + i keeps entry 8*g8 + i
    });
    // -- online softmax, one entry per lane; the denominator is summed per lane and reduced once at the end
    float corr[G];
    {
      const size_t xbase = ((size_t)((b * a.n_q + jq) * a.Hq + kvh * G)) * a.xs_stride + (size_t)(xs_tile0 + tile) * 64 + lane;
      float pv[GP];
#pragma unroll
      for (int h = 0; h < GP; ++h) pv[h] = 0.f;
      float x[G], xm[G];
#pragma unroll
      for (int h = 0; h < G; ++h) {
        x[h] = valid ? xt[h] * a.softmax_scale : -INFINITY;
        if (valid) a.xs[xbase + (size_t)h * a.xs_stride] = x[h];
        xm[h] = x[h];
      }
      wave_max_all<G>(xm);
#pragma unroll
      for (int h = 0; h < G; ++h) {
        // m_run starts at -inf and every tile has a live entry, so the first tile needs no special case:
        // corr = exp2(-inf) = 0 there, against zero accumulators
        const float mn = fmaxf(m_run[h], rdlane(xm[h], 63));
        corr[h] = __builtin_amdgcn_exp2f((m_run[h] - mn) * LOG2E);
        const float p = valid ? __builtin_amdgcn_exp2f((x[h] - mn) * LOG2E) : 0.f;
        l_lane[h] = fmaf(l_lane[h], corr[h], p);
        m_run[h] = mn;
        pv[h] = p;
      }
      static_for<GP / 4>([&](auto cc) {
        constexpr int c = decltype(cc)::value;
        u32x4 t;
        t.x = __builtin_bit_cast(uint32_t, pv[4 * c]); t.y = __builtin_bit_cast(uint32_t, pv[4 * c + 1]);
        t.z = __builtin_bit_cast(uint32_t, pv[4 * c + 2]); t.w = __builtin_bit_cast(uint32_t, pv[4 * c + 3]);
        lds_wr128<c * 16>(p_wr, t);
      });
    }
    {
      // the running maxima are wave-uniform; once they have settled no head needs rescaling (x * 1.0f is exact)
      bool moved = false;
#pragma unroll
      for (int h = 0; h < G; ++h) moved = moved || (corr[h] != 1.0f);
      if (moved) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
          osub[h] *= corr[h];
#pragma unroll
          for (int e = 0; e < EV; ++e) o[h][e] *= corr[h];
        }
      }
    }
    // -- V scales of this tile
    __builtin_amdgcn_s_setprio(MORE ? 2 : 0);
    float vsc[LPRV];
    if constexpr (GE::IS_Q) {
      wait_vm<N_K + X * (1 + SCD) + N_V>();
      const uint32_t base = w.sva + (uint32_t)(gv * LPRV) * 4u + ((M == Q_INT4) ? (uint32_t)(rv >> 3) * 256u : 0u);
      u32x4 t[LPRV / 4];
      static_for<LPRV / 4>([&](auto cc) { constexpr int c = decltype(cc)::value; t[c] = lds_rd128<c * 16>(base); });
      lds_wait(); tie(t);
      if constexpr (MORE) issue_vscale();
#pragma unroll
      for (int it = 0; it < LPRV; ++it) {
        if constexpr (M == Q_INT8) vsc[it] = elem_f(t[it / 4], it % 4);
        else vsc[it] = half_of(elem(t[it / 4], it % 4), (rv >> 2) & 1);        // unit rv lies in group rv/4
      }
    }
    // -- V rows: a step that has been read is refilled with the next tile's K pieces that fall on its bytes
    VStep<D, G, M> vb[2];
    auto read_v = [&](auto ic, VStep<D, G, M>& dst) {
      constexpr int it = decltype(ic)::value;
      // younger than this step's pieces: the later V pieces, the V-scale fetches of this period, the K pieces so far
      wait_vm<N_V - 1 - ((it + 1) * VU - 1) + X * (SCD + (it * VSB) / KIB)>();
      static_for<VU>([&](auto uc) {
        constexpr int u = decltype(uc)::value;
        if constexpr (VS == 16) dst.u[u] = lds_rd128<(it * VU + u) * VIB>(v_rd);
        else dst.u[u] = lds_rd32<(it * VU + u) * VIB>(v_rd);
      });
      static_for<GP / 4>([&](auto cc) {
        constexpr int c = decltype(cc)::value;
        dst.p[c] = lds_rd128<it * GP * 4 + c * 16>(p_rd);
      });
    };
    read_v(std::integral_constant<int, 0>{}, vb[0]);
    static_for<NITV>([&](auto ic) {
      constexpr int it = decltype(ic)::value;
      lds_wait(); tie(vb[it & 1].u); tie(vb[it & 1].p);
      if constexpr (MORE) {
#pragma unroll
        for (int s = (it * VSB) / KIB; s < ((it + 1) * VSB) / KIB; ++s) issue_k_piece(s);
      }
      if constexpr (it + 1 < NITV) read_v(std::integral_constant<int, (it + 1 < NITV ? it + 1 : NITV - 1)>{}, vb[(it + 1) & 1]);
      row_accumulate<D, G, M>(vb[it & 1], GE::IS_Q ? vsc[it] : 0.f, o, osub);
    });
    par ^= 1;
  };

  int tile = tile0;
  for (; (tile + tstride) * 64 < n_list; tile += tstride) tile_body(tile, std::true_type{});
  tile_body(tile, std::false_type{});

  if constexpr (GE::IS_Q) {
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < EV; ++e) o[h][e] = fmaf(-GE::OFF, osub[h], o[h][e]);
  }
}

// ---- one wave on the matrix cores: tiles of list F with 16-bit rows ------------------------------------------------
// The G query heads of the kv head are padded to the 16 columns of a 16x16x32 matrix instruction.
//   logits  : C[entry][head] = K[entry][:] . q[head][:], 16 entries per instruction, D/32 instructions deep.  Lane
//             (head = lane % 16, kb = lane / 16) ends up with the logits of entries 16*rb + 4*kb + 0..3 of its head,
//             which is exactly the layout of the left operand of the second product, so the probabilities never leave
//             the registers.
//   softmax : online per head; a lane's 16 entries of a tile, the maximum completed over the 4 lanes of the head.
//   output  : O[head][d] += P[head][entry] * V[entry][d], 32 entries per instruction; the right operand needs, per
//             lane, the same column of 4 + 4 rows: a transposing LDS read delivers it.  P is fed as two 16-bit terms
//             (leading bits and remainder), so the product carries 16 significant bits of every weight.
// Rows still come in by direct-to-LDS loads of 1 KB (8 rows x 8 pieces of 16 bytes, 128 contiguous bytes per row).
// Within a row's 128 bytes the pieces are rotated by an amount that depends on the row, so that the 16 lanes of an
// operand read (16 different rows, same piece) fall on 16 different bank groups; the rotation is undone by the read
// addresses.  K rows of a tile, its V rows and the next tile's K rows pass through the one tile buffer as in attn_wave:
// the K rows of 16 entries are replaced by V pieces once read, half a tile of V rows by the next tile's K pieces.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

template <int KT>
__device__ __forceinline__ f32x4 mfma_16x16x32(const u32x4& x, const u32x4& y, f32x4 c) {
  if constexpr (KT == KT_BF16)
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x), __builtin_bit_cast(bf16x8, y), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, x), __builtin_bit_cast(f16x8, y), c, 0, 0, 0);
}
// value of lane (lane ^ MASK)
template <int MASK>
__device__ __forceinline__ float lane_xor(float x, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane ^ MASK) << 2, __builtin_bit_cast(int, x)));
}
// A binary32 weight as a sum of 16-bit terms, each the leading bits (by truncation) of what the terms before it left.
// bfloat16: three terms of 8 significant bits are the weight exactly.  binary16: two terms of 11 bits (22 of the 24);
// the weights are taken times 2^P_SHIFT there, so that small ones stay clear of binary16's narrow exponent range
// (the factor is taken out of the accumulators at the end).
template <int KT>
struct PSplit {
  static constexpr int N = KT == KT_BF16 ? 3 : 2;
  static constexpr float P_SHIFT = KT == KT_BF16 ? 0.f : 14.f;
};
template <int KT>
__device__ __forceinline__ void split_pair(float p0, float p1, uint32_t (&t)[PSplit<KT>::N]) {
  if constexpr (KT == KT_BF16) {
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      const uint32_t u0 = __builtin_bit_cast(uint32_t, p0) & 0xffff0000u, u1 = __builtin_bit_cast(uint32_t, p1) & 0xffff0000u;
      t[i] = u1 | (u0 >> 16);
      p0 -= __builtin_bit_cast(float, u0);
      p1 -= __builtin_bit_cast(float, u1);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const f16x2 h = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(p0, p1));
      t[i] = __builtin_bit_cast(uint32_t, h);
      p0 -= (float)h.x;
      p1 -= (float)h.y;
    }
  }
}

// 16 code values (one byte each, or two per byte) as 16-bit floating point: the matrix cores multiply them exactly
// (a code + 128, or + 8, has at most 8 significant bits).  Two values per 32-bit word, low element first.
template <int KT>
__device__ __forceinline__ uint32_t pack16(float lo, float hi) {
  if constexpr (KT == KT_BF16) return __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, hi), __builtin_bit_cast(uint32_t, lo), 0x07060302u);
  else return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}
__device__ __forceinline__ float ubyte_f(uint32_t w, int n) {    // byte n of w as a float (one conversion instruction)
  return (float)((w >> (8 * n)) & 0xFFu);
}
// one word of int8 codes (4, as code + 128) -> two words; one word of int4 codes (8, as code + 8) -> four words
template <int KT>
__device__ __forceinline__ void widen_int8(uint32_t w, uint32_t& o0, uint32_t& o1) {
  w ^= 0x80808080u;
  o0 = pack16<KT>(ubyte_f(w, 0), ubyte_f(w, 1));
  o1 = pack16<KT>(ubyte_f(w, 2), ubyte_f(w, 3));
}
template <int KT>
__device__ __forceinline__ u32x4 widen_int4(uint32_t w) {
  w ^= 0x88888888u;
  const uint32_t lo = w & 0x0f0f0f0fu, hi = (w >> 4) & 0x0f0f0f0fu;    // elements 0, 2, 4, 6 and 1, 3, 5, 7
  return u32x4{pack16<KT>(ubyte_f(lo, 0), ubyte_f(hi, 0)), pack16<KT>(ubyte_f(lo, 1), ubyte_f(hi, 1)),
               pack16<KT>(ubyte_f(lo, 2), ubyte_f(hi, 2)), pack16<KT>(ubyte_f(lo, 3), ubyte_f(hi, 3))};
}

// M: F_BF16 / F_F16 (list F; the element type is KT's) or Q_INT8 / Q_INT4 (list Q).  NCB: blocks of 16 columns; a
// column is one (query token, head of the group) pair, query-major, a.cq query tokens in all (a decode step: one).
// Code rows (list Q) are fetched as they are stored (16-byte pieces, consecutive lanes along a row), and half a tile at
// a time is widened to 16-bit values of code + OFF into the free upper half of the wave's tile buffer, in the layout the
// full-precision rows arrive in, where the same operand reads pick it up.  Scales stay outside the products: a K row's
// scale multiplies its logits (per 32-element group: one product per group), a V row's scale its weights; the offset
// comes out through the sums of the query elements and of the scaled weights.
template <int D, int G, int KT, Mode M, int NCB>
__device__ __forceinline__ void attn_wave_mfma(const AttnArgs& a, const WaveLds& w, int b, int jz, int kvh, int lane,
                                               int tile0, int tstride, int n_list, const int* loc_list, int xs_tile0,
                                               f32x4 (&o)[NCB][D / 16], float (&m_run)[NCB], float (&l_run)[NCB]) {
  static_assert(KT == KT_BF16 || KT == KT_F16, "16-bit operands");
  static_assert(D % 64 == 0, "head_dim in whole 128-byte row halves");
  constexpr bool IS_Q = (M == Q_INT8 || M == Q_INT4);
  constexpr int RB = 2 * D;                    // bytes per row as the matrix cores read it
  constexpr int KU = RB / 128;                 // 1 KB pieces per batch of 8 rows (operand layout)
  constexpr int NKS = D / 32, NDB = D / 16;    // instructions deep (logits), output column blocks
  constexpr int PB = 1024;
  constexpr int CRB = !IS_Q ? RB : (M == Q_INT8 ? D : D / 2);   // bytes per row as fetched
  constexpr int NP = IS_Q ? CRB / 16 : 8 * KU;                  // 1 KB pieces per tile, K or V
  constexpr int NPH = NP / 2;
  constexpr int LPR = CRB / 16, RPP = 64 / LPR;                 // list Q: lanes per row, rows per piece
  constexpr int SCD = (M == Q_INT8) ? 1 : (M == Q_INT4) ? D / 64 : 0;   // dwords of scales per row
  constexpr int NGD = (M == Q_INT4) ? D / 32 : 1;               // scale groups along a row
  constexpr float OFF = (M == Q_INT4) ? 8.f : 128.f;
  constexpr uint32_t SCR = IS_Q ? 32 * RB : 0;                  // where the widened half tile sits
  static_assert(NP >= 2 && (!IS_Q || 64 * CRB <= 32 * RB), "two halves; code rows leave the upper half of the buffer free");
  const int g = lane >> 3, r = lane & 7;       // F fetch side: row of a batch, piece of the row's 128 bytes
  const int n = lane & 15, kb = lane >> 4;     // operand side

  __amdgpu_buffer_rsrc_t rk, rvv, rsk, rsv;
  if constexpr (!IS_Q) {
    const size_t off = (size_t)(b * a.Hkv + kvh) * a.capF * RB;
    rk = make_rsrc(a.fpK + off, (uint32_t)a.capF * RB); rvv = make_rsrc(a.fpV + off, (uint32_t)a.capF * RB);
    rsk = rk; rsv = rvv;
  } else {
    const size_t rows = (size_t)(b * a.Hkv + kvh) * a.cap2;
    rk = make_rsrc(a.c2K + rows * a.cb, (uint32_t)a.cap2 * a.cb); rvv = make_rsrc(a.c2V + rows * a.cb, (uint32_t)a.cap2 * a.cb);
    rsk = make_rsrc(a.s2K + rows * a.sb, (uint32_t)a.cap2 * a.sb); rsv = make_rsrc(a.s2V + rows * a.sb, (uint32_t)a.cap2 * a.sb);
  }
  const __amdgpu_buffer_rsrc_t rl = make_rsrc(loc_list, (uint32_t)a.Nmax * 4u);
  if (tile0 * 64 >= n_list) return;

  // the first tile's slot list before anything else (requests are served in the order they were made)
  dma<4>(rl, w.lt, (uint32_t)(tile0 * 64 + lane) * 4u, 0);

  // columns of this lane: (query token, head); right operand of the logits: elements 32*ks + 8*kb .. +7 of the
  // column's query vector (zeros for a column past the last)
  const int ncol = a.cq * G;
  bool live[NCB];
  int n_seen[NCB];                             // list entries the column's query may see (the chunk's later tokens are cut off list F)
  size_t xrow[NCB];
  u32x4 qreg[NCB][NKS];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int col = 16 * cb + n, jq = col / G, h = col % G;
    live[cb] = col < ncol;
    n_seen[cb] = IS_Q ? n_list : n_list - (live[cb] ? a.cq - 1 - jq : 0);
    const int qi = live[cb] ? jq * a.Hq + kvh * G + h : kvh * G;
    xrow[cb] = ((size_t)((b * a.n_q + jz) * a.cq * a.Hq + qi)) * a.xs_stride + (size_t)(4 * kb);
    const u32x4* qp = (const u32x4*)((const char*)a.q + (((size_t)b * a.q_bs + (size_t)jz * a.cq * a.Hq + qi) * D + 8 * kb) * 2);
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qreg[cb][ks] = live[cb] ? qp[ks * 4] : u32x4{0u, 0u, 0u, 0u};
  }

  // F fetch side.  Batch i holds entries 8*i + g; its K rows are rotated by 2*(g/2) + (i & 1) pieces, its V rows by g & 6.
  const uint32_t kcol0 = (uint32_t)((r + 2 * (g >> 1)) & 7) * 16u, kcol1 = (uint32_t)((r + 2 * (g >> 1) + 1) & 7) * 16u;
  const uint32_t vcol = (uint32_t)((r + (g & 6)) & 7) * 16u;
  // operand side.  Logits: lane (n, kb) reads piece 4*ks + kb of entry 16*rb + n, which is row n & 7 of batch
  // 2*rb + n/8; one address per parity of ks, the rest are immediates.
  uint32_t k_rd[2];
  {
    const int ii = n >> 3, gg = n & 7, rot = 2 * (gg >> 1) + ii;
#pragma unroll
    for (int par = 0; par < 2; ++par)
      k_rd[par] = w.ta + SCR + (uint32_t)(ii * KU * PB) + (uint32_t)(8 * gg + ((4 * par + kb - rot) & 7)) * 16u;
  }
  // Output: in the 16 lanes of block kb, lane 4*jj + q points at elements 4*q .. 4*q+3 of column block db of entry
  // 16*rb + 4*kb + jj (row 4*(kb & 1) + jj of batch 2*rb + kb/2); one address per db & 3
  uint32_t v_rd[4];
  {
    const int jj = (lane >> 2) & 3, qq = lane & 3, ii = kb >> 1, gg = 4 * (kb & 1) + jj;
#pragma unroll
    for (int dl = 0; dl < 4; ++dl)
      v_rd[dl] = w.ta + SCR + (uint32_t)(ii * KU * PB) + (uint32_t)(8 * gg + ((2 * dl - (gg & 6)) & 7) + (qq >> 1)) * 16u + (uint32_t)(qq & 1) * 8u;
  }
  // list Q: the lane's piece of a code row is widened and stored where the operand reads expect it.  Piece sl of a
  // half tile holds the half's entries RPP*sl + lane/LPR; the lane's 16 bytes are CPL 16-byte pieces of the wide row.
  constexpr int CPL = IS_Q ? RB / CRB : 1;
  auto wide_addr = [&](int sl, int k, bool v_side) -> uint32_t {
    const int el = RPP * sl + lane / LPR, i = el >> 3, gg = el & 7, cc = (lane % LPR) * CPL + k;
    const int rot = v_side ? (gg & 6) : 2 * (gg >> 1) + (i & 1);
    return w.ta + SCR + (uint32_t)((i * KU + (cc >> 3)) * PB) + (uint32_t)(8 * gg + (((cc & 7) - rot) & 7)) * 16u;
  };

  constexpr int NLK = IS_Q ? NP : 8;
  int lk[NLK], lrow = 0;                       // slots of the rows this lane fetches next (K side), and of entry `lane`
  auto read_locs = [&](int par, int nvalid) {
    const uint32_t base = w.lta + (uint32_t)par * 256u;
    if (nvalid < 64) {                                   // wave-uniform: a list's last tile
      if (lane >= nvalid) lds_wr32(base + (uint32_t)lane * 4u, 0xffffffffu);   // no row: fetches land as zeros
    }
    uint32_t t[NLK], me = 0;
    if constexpr (!IS_Q) {
      static_for<8>([&](auto ic) { constexpr int i = decltype(ic)::value; t[i] = lds_rd32<i * 32>(base + (uint32_t)g * 4u); });
    } else {
      static_for<NP>([&](auto ic) { constexpr int i = decltype(ic)::value; t[i] = lds_rd32<i * RPP * 4>(base + (uint32_t)(lane / LPR) * 4u); });
      me = lds_rd32<0>(base + (uint32_t)lane * 4u);
    }
    lds_wait(); tie(t); tie(me);
#pragma unroll
    for (int i = 0; i < NLK; ++i) lk[i] = (int)t[i];
    lrow = (int)me;
  };
  auto issue_loc = [&](int par, int tile) { dma<4>(rl, w.lt + par * 256, (uint32_t)(tile * 64 + lane) * 4u, 0); };
  auto issue_scales = [&]() {                            // K scales, then V scales, of the entry `lane`
#pragma unroll
    for (int j = 0; j < SCD; ++j) dma<4>(rsk, w.sk + j * 256, (uint32_t)lrow * (uint32_t)a.sb + j * 4u, 0);
#pragma unroll
    for (int j = 0; j < SCD; ++j) dma<4>(rsv, w.sv + j * 256, (uint32_t)lrow * (uint32_t)a.sb + j * 4u, 0);
  };
  auto issue_k_piece = [&](int s) {
    if constexpr (!IS_Q) {                               // (batch s / KU, row half s % KU)
      const int i = s / KU, j = s % KU;
      dma<16>(rk, w.t + s * PB, (uint32_t)lk[i] * (uint32_t)RB + (uint32_t)j * 128u + ((i & 1) ? kcol1 : kcol0), 1);
    } else {
      dma<16>(rk, w.t + s * PB, (uint32_t)lk[s] * (uint32_t)CRB + (uint32_t)(lane % LPR) * 16u, 1);
    }
  };

  wait_vm<0>();                                          // the list is in (and the query vectors)
  read_locs(0, n_list - tile0 * 64);
  issue_loc(1, tile0 + tstride);
  issue_scales();
#pragma unroll
  for (int s = 0; s < NP; ++s) issue_k_piece(s);

  // sums of the query elements, per scale group (the codes' offset comes out through them): a product with ones
  float qsum[NCB][NGD];
  if constexpr (IS_Q) {
    const uint32_t one2 = KT == KT_BF16 ? 0x3f803f80u : 0x3c003c00u;
    const u32x4 ones = u32x4{one2, one2, one2, one2};
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      float tot = 0.f;
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        const f32x4 s4 = mfma_16x16x32<KT>(ones, qreg[cb][ks], f32x4{0.f, 0.f, 0.f, 0.f});
        if constexpr (M == Q_INT4) qsum[cb][ks] = s4[0]; else tot += s4[0];
      }
      if constexpr (M == Q_INT8) qsum[cb][0] = tot;
    }
  }
  float osub[NCB][NGD];                                  // sums of the scaled weights, per lane (list Q)
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int gd = 0; gd < NGD; ++gd) osub[cb][gd] = 0.f;

  int par = 1;                                           // LDS half that holds the next tile's slot list
  auto tile_body = [&](int tile, auto more_c) {
    constexpr bool MORE = decltype(more_c)::value;
    constexpr int X = MORE ? 1 : 0;
    __builtin_amdgcn_s_setprio(MORE ? 3 : 1);
    int lv[NLK];                                         // this tile's V rows are fetched from the same slots
#pragma unroll
    for (int i = 0; i < NLK; ++i) lv[i] = lk[i];
    auto issue_v_piece = [&](int v) {
      if constexpr (!IS_Q) {
        const int i = v / KU, j = v % KU;
        dma<16>(rvv, w.t + v * PB, (uint32_t)lv[i] * (uint32_t)RB + (uint32_t)j * 128u + vcol, 1);
      } else {
        dma<16>(rvv, w.t + v * PB, (uint32_t)lv[v] * (uint32_t)CRB + (uint32_t)(lane % LPR) * 16u, 1);
      }
    };
    if constexpr (MORE) {
      wait_vm<2 * SCD + NP>();                           // younger than the next list: this tile's scales and K pieces
      read_locs(par, n_list - (tile + tstride) * 64);
      issue_loc(par ^ 1, tile + 2 * tstride);
    }
    // -- logits, 16 entries at a time
    f32x4 c[NCB][4];
    auto logits_of = [&](auto rc, const u32x4 (&ka)[NKS]) {    // rc: the 16-entry block
      constexpr int rb = decltype(rc)::value;
      if constexpr (M == Q_INT4) {
        // one product per scale group; the four entries' scales of dword ks/2, half ks & 1
        u32x4 sc[SCD];
        static_for<SCD>([&](auto jc) { constexpr int j = decltype(jc)::value; sc[j] = lds_rd128<j * 256 + rb * 64>(w.ska + (uint32_t)kb * 16u); });
        lds_wait(); tie(sc);
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
          f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < NKS; ++ks) {
            const f32x4 part = mfma_16x16x32<KT>(ka[ks], qreg[cb][ks], f32x4{0.f, 0.f, 0.f, 0.f});
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = fmaf(half_of(elem(sc[ks >> 1], j), ks & 1), fmaf(-OFF, qsum[cb][ks], part[j]), acc[j]);
          }
          c[cb][rb] = acc;
        }
      } else {
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
          f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < NKS; ++ks) acc = mfma_16x16x32<KT>(ka[ks], qreg[cb][ks], acc);
          c[cb][rb] = acc;
        }
        if constexpr (M == Q_INT8) {
          u32x4 sc = lds_rd128<rb * 64>(w.ska + (uint32_t)kb * 16u);
          lds_wait(); tie(sc);
#pragma unroll
          for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int j = 0; j < 4; ++j) c[cb][rb][j] = elem_f(sc, j) * fmaf(-OFF, qsum[cb][0], c[cb][rb][j]);
        }
      }
    };
    if constexpr (!IS_Q) {
      // the K rows of 16 entries that have been read are replaced by V pieces
      u32x4 ka[2][NKS];
      auto read_k = [&](auto rc, u32x4 (&dst)[NKS]) {
        constexpr int rb = decltype(rc)::value;
        // younger than these K pieces: the later K pieces, this period's list fetch, the V pieces so far
        wait_vm<NP - 2 * KU + X>();
        static_for<NKS>([&](auto kc) {
          constexpr int ks = decltype(kc)::value;
          dst[ks] = lds_rd128<(rb * 2 * KU + (ks >> 1)) * PB>(k_rd[ks & 1]);
        });
      };
      read_k(std::integral_constant<int, 0>{}, ka[0]);
      static_for<4>([&](auto rc) {
        constexpr int rb = decltype(rc)::value;
        lds_wait(); tie(ka[rb & 1]);
#pragma unroll
        for (int v = 2 * rb * KU; v < (2 * rb + 2) * KU; ++v) issue_v_piece(v);
        if constexpr (rb + 1 < 4) read_k(std::integral_constant<int, (rb + 1 < 4 ? rb + 1 : 3)>{}, ka[(rb + 1) & 1]);
        logits_of(rc, ka[rb & 1]);
      });
    } else {
      // half a tile of code rows is widened, then replaced by V pieces
      static_for<2>([&](auto hc) {
        constexpr int hf = decltype(hc)::value;
        // younger than this half's K pieces: the other half's, this period's list fetch, the V pieces so far
        wait_vm<NP - NPH + X>();
        u32x4 cu[NPH];
        static_for<NPH>([&](auto sc) { constexpr int sl = decltype(sc)::value; cu[sl] = lds_rd128<(hf * NPH + sl) * PB>(w.ta + (uint32_t)lane * 16u); });
        lds_wait(); tie(cu);
#pragma unroll
        for (int v = hf * NPH; v < (hf + 1) * NPH; ++v) issue_v_piece(v);
#pragma unroll
        for (int sl = 0; sl < NPH; ++sl) {
          if constexpr (M == Q_INT8) {
#pragma unroll
            for (int k = 0; k < 2; ++k) {
              uint32_t w0, w1, w2, w3;
              widen_int8<KT>(elem(cu[sl], 2 * k), w0, w1);
              widen_int8<KT>(elem(cu[sl], 2 * k + 1), w2, w3);
              lds_wr128<0>(wide_addr(sl, k, false), u32x4{w0, w1, w2, w3});
            }
          } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) lds_wr128<0>(wide_addr(sl, k, false), widen_int4<KT>(elem(cu[sl], k)));
          }
        }
        static_for<2>([&](auto rlc) {
          constexpr int rl2 = decltype(rlc)::value;
          u32x4 ka[NKS];
          static_for<NKS>([&](auto kc) {
            constexpr int ks = decltype(kc)::value;
            ka[ks] = lds_rd128<(rl2 * 2 * KU + (ks >> 1)) * PB>(k_rd[ks & 1]);
          });
          lds_wait(); tie(ka);
          logits_of(std::integral_constant<int, 2 * hf + rl2>{}, ka);
        });
      });
    }
    // -- online softmax: the lane has entries 16*rb + 4*kb + j of its column
    float p[NCB][4][4];
    {
      const int e0 = tile * 64 + 4 * kb;
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        float mx = -INFINITY;
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) {
          f32x4 x;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            x[j] = (e0 + 16 * rb + j < n_seen[cb]) ? c[cb][rb][j] * a.softmax_scale : -INFINITY;
            p[cb][rb][j] = x[j];
            mx = fmaxf(mx, x[j]);
          }
          if (live[cb]) *(f32x4*)(a.xs + xrow[cb] + (size_t)(xs_tile0 + tile) * 64 + 16 * rb) = x;
        }
        mx = fmaxf(mx, lane_xor<16>(mx, lane));
        mx = fmaxf(mx, lane_xor<32>(mx, lane));
        // m_run starts at -inf: corr = exp2(-inf) = 0 against zero accumulators.  A tile of which the column sees
        // nothing (an early token of a chunk, the list's last tile) leaves mn at -inf: nothing to add, nothing to rescale.
        const float mn = fmaxf(m_run[cb], mx);
        const float corr = mn > -INFINITY ? __builtin_amdgcn_exp2f((m_run[cb] - mn) * LOG2E) : 1.0f;
        float ps = 0.f;
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            p[cb][rb][j] = mn > -INFINITY ? __builtin_amdgcn_exp2f(fmaf(p[cb][rb][j] - mn, LOG2E, PSplit<KT>::P_SHIFT)) : 0.f;
            ps += p[cb][rb][j];
          }
        l_run[cb] = fmaf(l_run[cb], corr, ps);
        m_run[cb] = mn;
#pragma unroll
        for (int gd = 0; gd < NGD; ++gd) osub[cb][gd] *= corr;
        // the output accumulators of this lane belong to columns 4*kb + j: their factors come from those columns'
        // lanes; once the maxima have settled nothing needs rescaling (x * 1.0f is exact)
        if (__builtin_amdgcn_ballot_w64(corr != 1.0f) != 0) {
          float cj[4];
#pragma unroll
          for (int j = 0; j < 4; ++j)
            cj[j] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((4 * kb + j) << 2, __builtin_bit_cast(int, corr)));
#pragma unroll
          for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int j = 0; j < 4; ++j) o[cb][db][j] *= cj[j];
        }
      }
    }
    // -- output: 32 entries per instruction; half a tile of V rows that has been read is replaced by K pieces
    __builtin_amdgcn_s_setprio(MORE ? 2 : 0);
    constexpr int NT = PSplit<KT>::N;
    // V scales of the tile: the 4 entries' of each 16-entry block (all older than the K pieces: they are in)
    u32x4 vsc[IS_Q ? SCD : 1][4];
    if constexpr (IS_Q) {
      static_for<SCD>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        static_for<4>([&](auto rc) { constexpr int rb = decltype(rc)::value; vsc[j][rb] = lds_rd128<j * 256 + rb * 64>(w.sva + (uint32_t)kb * 16u); });
      });
      lds_wait();
#pragma unroll
      for (int j = 0; j < SCD; ++j) tie(vsc[j]);
      if constexpr (MORE) issue_scales();                // both scale regions are free: the next tile's
    }
    // weights of the half's 32 entries as operand terms; list Q: times the V row's scale (of scale group gd)
    auto weights = [&](auto tc, int cb, int gd, u32x4 (&pt)[NT]) {
      constexpr int t = decltype(tc)::value;
      float pw[2][4];
#pragma unroll
      for (int r2 = 0; r2 < 2; ++r2)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float v = p[cb][2 * t + r2][j];
          if constexpr (M == Q_INT8) v *= elem_f(vsc[0][2 * t + r2], j);
          if constexpr (M == Q_INT4) v *= half_of(elem(vsc[gd >> 1][2 * t + r2], j), gd & 1);
          if constexpr (IS_Q) osub[cb][gd] += v;
          pw[r2][j] = v;
        }
      uint32_t s0[NT], s1[NT], s2[NT], s3[NT];
      split_pair<KT>(pw[0][0], pw[0][1], s0);
      split_pair<KT>(pw[0][2], pw[0][3], s1);
      split_pair<KT>(pw[1][0], pw[1][1], s2);
      split_pair<KT>(pw[1][2], pw[1][3], s3);
#pragma unroll
      for (int i = 0; i < NT; ++i) pt[i] = u32x4{s0[i], s1[i], s2[i], s3[i]};
    };
    static_for<2>([&](auto tc) {
      constexpr int t = decltype(tc)::value;
      // younger than this half's V pieces: the other half's, the next tile's scales, the K pieces issued after the first half
      wait_vm<NPH * (1 - t) + X * (2 * SCD + t * NPH)>();
      if constexpr (IS_Q) {
        u32x4 cu[NPH];
        static_for<NPH>([&](auto sc) { constexpr int sl = decltype(sc)::value; cu[sl] = lds_rd128<(t * NPH + sl) * PB>(w.ta + (uint32_t)lane * 16u); });
        lds_wait(); tie(cu);
        if constexpr (MORE) {
#pragma unroll
          for (int s = t * NPH; s < (t + 1) * NPH; ++s) issue_k_piece(s);
        }
#pragma unroll
        for (int sl = 0; sl < NPH; ++sl) {
          if constexpr (M == Q_INT8) {
#pragma unroll
            for (int k = 0; k < 2; ++k) {
              uint32_t w0, w1, w2, w3;
              widen_int8<KT>(elem(cu[sl], 2 * k), w0, w1);
              widen_int8<KT>(elem(cu[sl], 2 * k + 1), w2, w3);
              lds_wr128<0>(wide_addr(sl, k, true), u32x4{w0, w1, w2, w3});
            }
          } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) lds_wr128<0>(wide_addr(sl, k, true), widen_int4<KT>(elem(cu[sl], k)));
          }
        }
      }
      constexpr int RB0 = IS_Q ? 0 : 2 * t;              // the widened half sits at the start of its area
      u32x2 vv[2][NDB];
      static_for<2>([&](auto r2c) {
        constexpr int r2 = decltype(r2c)::value;
        static_for<NDB>([&](auto dc) {
          constexpr int db = decltype(dc)::value;
          vv[r2][db] = lds_rd64_tr16<((RB0 + r2) * 2 * KU + (db >> 2)) * PB>(v_rd[db & 3]);
        });
      });
      lds_wait(); tie(vv[0]); tie(vv[1]);
      if constexpr (!IS_Q && MORE) {
#pragma unroll
        for (int s = t * NPH; s < (t + 1) * NPH; ++s) issue_k_piece(s);
      }
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        u32x4 pt[NT];
        if constexpr (M != Q_INT4) weights(tc, cb, 0, pt);
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          if constexpr (M == Q_INT4) { if (db % 2 == 0) weights(tc, cb, db / 2, pt); }
          const u32x4 vb = u32x4{vv[0][db].x, vv[0][db].y, vv[1][db].x, vv[1][db].y};
#pragma unroll
          for (int i = NT - 1; i >= 0; --i) o[cb][db] = mfma_16x16x32<KT>(pt[i], vb, o[cb][db]);
        }
      }
    });
    par ^= 1;
  };

  int tile = tile0;
  for (; (tile + tstride) * 64 < n_list; tile += tstride) tile_body(tile, std::true_type{});
  tile_body(tile, std::false_type{});

  if constexpr (IS_Q) {
    // the codes went in as code + OFF: take OFF times the sum of the scaled weights back out, per column (the
    // accumulators of this lane belong to columns 4*kb + j)
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int gd = 0; gd < NGD; ++gd) {
        float s = osub[cb][gd];
        s += lane_xor<16>(s, lane);
        s += lane_xor<32>(s, lane);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float sj = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((4 * kb + j) << 2, __builtin_bit_cast(int, s)));
#pragma unroll
          for (int db = 0; db < NDB; ++db)
            if (NGD == 1 || db / 2 == gd) o[cb][db][j] = fmaf(-OFF, sj, o[cb][db][j]);
        }
      }
  }
  if constexpr (PSplit<KT>::P_SHIFT != 0.f) {
    const float back = __builtin_amdgcn_exp2f(-PSplit<KT>::P_SHIFT);
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      l_run[cb] *= back;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int j = 0; j < 4; ++j) o[cb][db][j] *= back;
    }
  }
}

// Waves per SIMD the kernel is compiled for: two while a wave's registers (query slices and output accumulators grow
// with the group size) fit half a SIMD's file, else one.
constexpr int waves_per_simd(int G) { return G <= 5 ? 2 : 1; }
// One workgroup per compute unit: as many waves as the register budget allows (4 SIMDs) and as fit the LDS with a
// whole-tile buffer each (64 rows: 16 KB at 256-byte rows, 32 KB at 512-byte rows).
constexpr int waves_per_group(int row_bytes, int G) {
  return (row_bytes > 256 && waves_per_simd(G) * 4 > 4) ? 4 : waves_per_simd(G) * 4;
}

template <int D, int G, int KT>
struct KernelGeo {
  static constexpr Mode MF = KT == KT_BF16 ? F_BF16 : KT == KT_F16 ? F_F16 : F_F32;
  static constexpr int RB = Geo<D, MF>::RB;
  static constexpr int NW = waves_per_group(RB, G);
  static constexpr int EV = Geo<D, MF>::EV;
  static constexpr int LPRV = Geo<D, MF>::LPRV;
};

// Waves of a (sequence, kv head) pair that serve the Q list, out of nwv, for nft F tiles and nqt Q tiles: the split
// that minimises the longest wave.  A code tile moves fewer bytes than a full-precision one but costs more vector
// instructions (unpacking); it is priced QCOST_Q against QCOST_F for an F tile.  Depends on the list lengths only.
constexpr int QCOST_F = 4, QCOST_Q = 5;
__host__ __device__ inline int q_waves(int nwv, int nft, int nqt) {
  if (nqt == 0) return 0;
  if (nft == 0) return nwv;
  int best = 1, best_cost = 0x7fffffff;
  for (int n = 1; n < nwv; ++n) {
    const int cf = ((nft + (nwv - n) - 1) / (nwv - n)) * QCOST_F, cq = ((nqt + n - 1) / n) * QCOST_Q;
    const int c = cf > cq ? cf : cq;
    if (c < best_cost) { best_cost = c; best = n; }
  }
  return best;
}

template <int D, int G, int KT>
__global__ __launch_bounds__((KernelGeo<D, G, KT>::NW * 64), (KernelGeo<D, G, KT>::NW / 4)) void k_attn_tiered(const AttnArgs a) {
  using KG = KernelGeo<D, G, KT>;
  constexpr int NW = KG::NW, EV = KG::EV, LPRV = KG::LPRV, GP = GPad<G>::v;
  constexpr int TILE_BYTES = 64 * KG::RB;
  static_assert(G * D * 4 <= TILE_BYTES, "a wave's output partial is parked in its tile buffer");
  __shared__ __attribute__((aligned(16))) char sm_t[NW * TILE_BYTES];
  __shared__ __attribute__((aligned(16))) char sm_sc[NW * 2 * 512];
  __shared__ __attribute__((aligned(16))) char sm_lt[NW * 512];
  __shared__ __attribute__((aligned(16))) float sm_p[NW * 64 * GP];
  __shared__ float sm_ml[NW * 16];
  // A wave's row groups (64 / LPRV of them) each hold a partial sum of every output element.  As many of them as the
  // tile buffer has room for are parked side by side and added up by the merge below; only if there are more (64-byte
  // rows) are the upper ones first folded into the lower ones by shuffles.
  constexpr int NG = 64 / LPRV, FIT = TILE_BYTES / (G * D * 4);
  constexpr int NGK = NG <= FIT ? NG : (FIT >= 4 ? 4 : FIT >= 2 ? 2 : 1);
  const int s = blockIdx.x, kvh = blockIdx.y;
  // several query tokens per sequence: query jq of sequence b; it is n_q - 1 - jq positions older than the last one,
  // and those positions (the tail of list F) are not its to see
  const int b = a.n_q > 1 ? (int)blockIdx.z / a.n_q : (int)blockIdx.z, jq = a.n_q > 1 ? (int)blockIdx.z % a.n_q : 0;
  const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
  int nF, nQ, xsb = 0;
  if (!a.second) {
    if (a.B <= ATTN_ARG_SEQS) { nF = a.nF[b]; nQ = a.nQ[b]; }
    else { nF = a.cnt[b * CNT_N + C_NF] - a.trim; nQ = a.cnt[b * CNT_N + C_NQ]; }
    nF -= a.n_q - 1 - jq;
  } else {
    nF = a.cnt[b * CNT_N + C_NS]; nQ = 0;
    xsb = ((a.cnt[b * CNT_N + C_NF] - a.trim + 63) >> 6) + ((a.cnt[b * CNT_N + C_NQ] + 63) >> 6);
  }
  const int nft = (nF + 63) >> 6, nqt = (nQ + 63) >> 6;
  const int nwv = a.S * NW;
  const int nwq = a.second ? 0 : (a.B <= ATTN_ARG_SEQS && a.n_q == 1) ? a.nWq[b] : q_waves(nwv, nft, nqt), nwf = nwv - nwq;
  const int u = s * NW + wave;

  WaveLds w;
  w.t = sm_t + wave * TILE_BYTES;
  w.sk = sm_sc + wave * 1024; w.sv = w.sk + 512; w.lt = sm_lt + wave * 512;
  w.ta = lds_addr(w.t); w.ska = lds_addr(w.sk); w.sva = lds_addr(w.sv); w.lta = lds_addr(w.lt);
  w.p = (char*)(sm_p + wave * 64 * GP);
  w.pa = lds_addr(w.p);
  float* my_o = (float*)w.t;          // after the wave's last tile: its output partial, [G][D]

  float o[G][EV], m_run[G], l_lane[G];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    m_run[h] = -INFINITY; l_lane[h] = 0.f;
#pragma unroll
    for (int e = 0; e < EV; ++e) o[h][e] = 0.f;
  }
  bool o_written = false;
  if (u < nwf) {
    attn_wave<D, G, KG::MF, KT>(a, w, b, jq, kvh, lane, u, nwf, nF, a.f_loc + (size_t)b * a.Nmax, xsb, o, m_run, l_lane);
  } else {
    if constexpr (EV == 8) {
      if (a.t2fmt == 0) attn_wave<D, G, Q_INT8, KT>(a, w, b, jq, kvh, lane, u - nwf, nwq, nQ, a.q_loc + (size_t)b * a.Nmax, xsb + nft, o, m_run, l_lane);
      else attn_wave<D, G, Q_INT4, KT>(a, w, b, jq, kvh, lane, u - nwf, nwq, nQ, a.q_loc + (size_t)b * a.Nmax, xsb + nft, o, m_run, l_lane);
    } else {
      // binary32 rows use 4 elements per lane, code rows 8: separate accumulators, parked directly
      float o8[G][8];
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int e = 0; e < 8; ++e) o8[h][e] = 0.f;
      if (a.t2fmt == 0) attn_wave<D, G, Q_INT8, KT>(a, w, b, jq, kvh, lane, u - nwf, nwq, nQ, a.q_loc + (size_t)b * a.Nmax, xsb + nft, o8, m_run, l_lane);
      else attn_wave<D, G, Q_INT4, KT>(a, w, b, jq, kvh, lane, u - nwf, nwq, nQ, a.q_loc + (size_t)b * a.Nmax, xsb + nft, o8, m_run, l_lane);
      constexpr int L8 = D / 8;
#pragma unroll
      for (int st = L8; st < 64; st <<= 1)
#pragma unroll
        for (int h = 0; h < G; ++h)
#pragma unroll
          for (int e = 0; e < 8; ++e) o8[h][e] += __shfl_xor(o8[h][e], st);
      if (lane < L8) {
#pragma unroll
        for (int h = 0; h < G; ++h)
#pragma unroll
          for (int e = 0; e < 8; ++e) my_o[h * D + lane * 8 + e] = o8[h][e];
      }
      // the merge adds NGK parked row groups per wave: this wave has one, the others are zero
      for (int i = lane; i < (NGK - 1) * G * D; i += 64) my_o[G * D + i] = 0.f;
      o_written = true;
    }
  }
  // ---- wave partial: sum the row groups and the per-lane denominators, then merge the waves through LDS
  if (!o_written) {
#pragma unroll
    for (int st = LPRV * NGK; st < 64; st <<= 1)
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int e = 0; e < EV; ++e) o[h][e] += __shfl_xor(o[h][e], st);
    if (lane < LPRV * NGK) {
      float* dst = my_o + (lane / LPRV) * (G * D) + (lane % LPRV) * EV;
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int e = 0; e < EV; ++e) dst[h * D + e] = o[h][e];
    }
  }
#pragma unroll
  for (int h = 0; h < G; ++h) {
    const float ls = wave_sum(l_lane[h]);
    if (lane == 0) { sm_ml[wave * 16 + h] = m_run[h]; sm_ml[wave * 16 + 8 + h] = ls; }
  }
  __syncthreads();
  const int bq = b * a.n_q + jq;
  float* po = a.part_o + ((size_t)((bq * a.Hkv + kvh) * a.S_total + a.s0 + s) * G) * D;
  for (int i = t; i < G * D; i += NW * 64) {
    const int h = i / D;
    float mb = sm_ml[h];
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) mb = fmaxf(mb, sm_ml[ww * 16 + h]);
    float acc = 0.f;
    if (mb > -INFINITY) {
#pragma unroll
      for (int ww = 0; ww < NW; ++ww) {
        const float* src = (const float*)(sm_t + ww * TILE_BYTES) + i;
        float part = src[0];                                // the wave's row groups, in order
#pragma unroll
        for (int g = 1; g < NGK; ++g) part += src[g * (G * D)];
        acc = fmaf(__builtin_amdgcn_exp2f((sm_ml[ww * 16 + h] - mb) * LOG2E), part, acc);
      }
    }
    po[i] = acc;
  }
  if (t < G) {
    float mb = sm_ml[t];
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) mb = fmaxf(mb, sm_ml[ww * 16 + t]);
    float ll = 0.f;
    if (mb > -INFINITY) {
#pragma unroll
      for (int ww = 0; ww < NW; ++ww) ll = fmaf(__builtin_amdgcn_exp2f((sm_ml[ww * 16 + t] - mb) * LOG2E), sm_ml[ww * 16 + 8 + t], ll);
    }
    float* pm = a.part_ml + ((size_t)((bq * a.Hkv + kvh) * a.S_total + a.s0 + s) * 2) * G;
    pm[t] = mb;
    pm[G + t] = ll;
  }
}

// ---- the same launch for 16-bit rows: every wave on the matrix cores ------------------------------------------------
// Eight waves per workgroup whatever the group size (the accumulators are 16 columns wide either way), a 64-row tile
// buffer each; with a second block of 16 columns (chunks of query tokens) the registers allow four.  A wave's result
// arrives complete (no row-group partials): [column][D] parked in its tile buffer.
constexpr int mc_waves(int ncb) { return ncb == 1 ? 8 : 4; }
template <int D, int G, int KT, int NCB>
__global__ __launch_bounds__(mc_waves(NCB) * 64, mc_waves(NCB) / 4) void k_attn_tiered_mc(const AttnArgs a) {
  constexpr int NW = mc_waves(NCB), RB = 2 * D, TILE_BYTES = 64 * RB;
  constexpr Mode MF = KT == KT_BF16 ? F_BF16 : F_F16;
  static_assert(16 * NCB * D * 4 <= TILE_BYTES, "a wave's output partial is parked in its tile buffer");
  __shared__ __attribute__((aligned(16))) char sm_t[NW * TILE_BYTES];
  __shared__ __attribute__((aligned(16))) char sm_sc[NW * 2 * 512];
  __shared__ __attribute__((aligned(16))) char sm_lt[NW * 512];
  __shared__ float sm_ml[NW * 64];                       // per wave: m of 32 columns, then l
  const int s = blockIdx.x, kvh = blockIdx.y;
  // query tokens beyond one per sequence: a.cq of them as columns of this workgroup, a.n_q such groups along grid z.
  // The group's last token is (n_q - 1 - jz) * cq positions older than the chunk's last, and that many entries at the
  // end of list F are not the group's to see (its earlier tokens cut off more, column by column).
  const int b = a.n_q > 1 ? (int)blockIdx.z / a.n_q : (int)blockIdx.z, jz = a.n_q > 1 ? (int)blockIdx.z % a.n_q : 0;
  const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
  int nF, nQ, xsb = 0;
  if (!a.second) {
    if (a.B <= ATTN_ARG_SEQS) { nF = a.nF[b]; nQ = a.nQ[b]; }
    else { nF = a.cnt[b * CNT_N + C_NF] - a.trim; nQ = a.cnt[b * CNT_N + C_NQ]; }
    nF -= (a.n_q - 1 - jz) * a.cq;
  } else {
    nF = a.cnt[b * CNT_N + C_NS]; nQ = 0;
    xsb = ((a.cnt[b * CNT_N + C_NF] - a.trim + 63) >> 6) + ((a.cnt[b * CNT_N + C_NQ] + 63) >> 6);
  }
  const int nft = (nF + 63) >> 6, nqt = (nQ + 63) >> 6;
  const int nwv = a.S * NW;
  const int nwq = a.second ? 0 : (a.B <= ATTN_ARG_SEQS && a.n_q == 1) ? a.nWq[b] : q_waves(nwv, nft, nqt), nwf = nwv - nwq;
  const int u = s * NW + wave;
  const int ncol = a.cq * G;

  WaveLds w;
  w.t = sm_t + wave * TILE_BYTES;
  w.sk = sm_sc + wave * 1024; w.sv = w.sk + 512; w.lt = sm_lt + wave * 512;
  w.ta = lds_addr(w.t); w.ska = lds_addr(w.sk); w.sva = lds_addr(w.sv); w.lta = lds_addr(w.lt);
  w.p = nullptr; w.pa = 0;
  float* my_o = (float*)w.t;          // after the wave's last tile: its output partial, [column][D]

  f32x4 om[NCB][D / 16];
  float mr[NCB], lr[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    mr[cb] = -INFINITY; lr[cb] = 0.f;
#pragma unroll
    for (int db = 0; db < D / 16; ++db) om[cb][db] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  if (u < nwf) attn_wave_mfma<D, G, KT, MF, NCB>(a, w, b, jz, kvh, lane, u, nwf, nF, a.f_loc + (size_t)b * a.Nmax, xsb, om, mr, lr);
  else if (a.t2fmt == 0) attn_wave_mfma<D, G, KT, Q_INT8, NCB>(a, w, b, jz, kvh, lane, u - nwf, nwq, nQ, a.q_loc + (size_t)b * a.Nmax, xsb + nft, om, mr, lr);
  else attn_wave_mfma<D, G, KT, Q_INT4, NCB>(a, w, b, jz, kvh, lane, u - nwf, nwq, nQ, a.q_loc + (size_t)b * a.Nmax, xsb + nft, om, mr, lr);
  // ---- wave partial into LDS: lane (n, kb) has the statistics of column 16*cb + n and the outputs of columns
  // 16*cb + 4*kb + j, element 16*db + n
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    float ls = lr[cb];
    ls += lane_xor<16>(ls, lane);
    ls += lane_xor<32>(ls, lane);
    const int col = 16 * cb + lane;
    if (lane < 16 && col < ncol) { sm_ml[wave * 64 + col] = mr[cb]; sm_ml[wave * 64 + 32 + col] = ls; }
#pragma unroll
    for (int db = 0; db < D / 16; ++db)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = 16 * cb + 4 * (lane >> 4) + j;
        if (c < ncol) my_o[c * D + 16 * db + (lane & 15)] = om[cb][db][j];
      }
  }
  __syncthreads();
  // ---- merge the waves: one split partial (m, l, o[G][D]) per query token
  const int bq0 = (b * a.n_q + jz) * a.cq;
  for (int i = t; i < ncol * D; i += NW * 64) {
    const int col = i / D, d = i % D, jq = col / G, h = col % G;
    float mb = sm_ml[col];
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) mb = fmaxf(mb, sm_ml[ww * 64 + col]);
    float acc = 0.f;
    if (mb > -INFINITY) {
#pragma unroll
      for (int ww = 0; ww < NW; ++ww)
        acc = fmaf(__builtin_amdgcn_exp2f((sm_ml[ww * 64 + col] - mb) * LOG2E), ((const float*)(sm_t + ww * TILE_BYTES))[i], acc);
    }
    a.part_o[((size_t)(((bq0 + jq) * a.Hkv + kvh) * a.S_total + a.s0 + s) * G + h) * D + d] = acc;
  }
  if (t < ncol) {
    const int jq = t / G, h = t % G;
    float mb = sm_ml[t];
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) mb = fmaxf(mb, sm_ml[ww * 64 + t]);
    float ll = 0.f;
    if (mb > -INFINITY) {
#pragma unroll
      for (int ww = 0; ww < NW; ++ww) ll = fmaf(__builtin_amdgcn_exp2f((sm_ml[ww * 64 + t] - mb) * LOG2E), sm_ml[ww * 64 + 32 + t], ll);
    }
    float* pm = a.part_ml + ((size_t)(((bq0 + jq) * a.Hkv + kvh) * a.S_total + a.s0 + s) * 2) * G;
    pm[h] = mb;
    pm[G + h] = ll;
  }
}

// ---- finish: global softmax statistics, scores, output ------------------------------------------------------
constexpr int FIN_LDS_FLOATS = 2048;   // room for the (m, l) of all splits of one sequence, Hkv * S * 2 * G floats, in all but the smallest batches (else they are read from memory)

template <int D, int G>
__global__ __launch_bounds__(256) void k_attn_finish(const AttnArgs a, int n_tiles) {
  __shared__ float sm_pm[FIN_LDS_FLOATS];
  __shared__ float M[128], IL[128];
  const int t = threadIdx.x, b = blockIdx.y;
  int nF, nQ, nS;
  if (a.B <= ATTN_ARG_SEQS) { nF = a.nF[b]; nQ = a.nQ[b]; }
  else { nF = a.cnt[b * CNT_N + C_NF] - a.trim; nQ = a.cnt[b * CNT_N + C_NQ]; }
  nS = a.s_pos ? a.cnt[b * CNT_N + C_NS] : 0;
  // logits columns: F tiles, Q tiles, then (streamed T1) the T1 list's tiles
  const int cf = (nF + TB - 1) / TB, cq = (nQ + TB - 1) / TB, ns = a.S_total;
  const bool is_tile = (int)blockIdx.x < n_tiles;
  if (is_tile && (int)blockIdx.x * 64 >= (nS > 0 ? (cf + cq) * TB + nS : cf * TB + nQ)) return;
  // tile workgroups: the entry's position, its first kv head's logits and its score so far are fetched before the
  // (m, l) merge, so their latency runs beside it
  const int e = t & 63, hg = t >> 6;
  const int j = blockIdx.x * 64 + e;
  int pos = -1;
  float x0[G], score_old = 0.f;
  if (is_tile) {
    const bool in_f = j < nF, in_q = j >= cf * TB && j - cf * TB < nQ, in_s = j >= (cf + cq) * TB && j - (cf + cq) * TB < nS;
    const bool live = in_f || in_q || in_s;      // from the list lengths alone: the logits are fetched beside the position
    if (in_f) pos = a.f_pos[(size_t)b * a.Nmax + j];
    else if (in_q) pos = a.q_pos[(size_t)b * a.Nmax + (j - cf * TB)];
    else if (in_s) pos = a.s_pos[(size_t)b * a.Nmax + (j - (cf + cq) * TB)];
#pragma unroll
    for (int g = 0; g < G; ++g) x0[g] = (live && hg < a.Hkv) ? a.xs[((size_t)b * a.Hq + hg * G + g) * a.xs_stride + j] : 0.f;
    if (hg == 0 && pos >= 0) score_old = a.score[(size_t)b * a.Nmax + pos];
  }
  // (m, l) of every split of this sequence: part_ml[b][kvh][s][2][G], s < ns
  const float* pmb = a.part_ml + (size_t)b * a.Hkv * a.S_total * 2 * G;
  const int per_kvh = ns * 2 * G;
  const bool in_lds = a.Hkv * per_kvh <= FIN_LDS_FLOATS;
  if (in_lds) {
    for (int i = t; i < a.Hkv * per_kvh; i += 256) {
      const int kvh = i / per_kvh, rem = i % per_kvh;
      sm_pm[i] = pmb[(size_t)kvh * a.S_total * 2 * G + rem];
    }
    __syncthreads();
  }
  if (t < a.Hq) {
    const int kvh = t / G, g = t % G;
    const float* src = in_lds ? (sm_pm + kvh * per_kvh) : (pmb + (size_t)kvh * a.S_total * 2 * G);
    float mm = -INFINITY;
    for (int k = 0; k < ns; ++k) mm = fmaxf(mm, src[k * 2 * G + g]);
    float ll = 0.f;
    for (int k = 0; k < ns; ++k) ll = fmaf(src[k * 2 * G + G + g], __builtin_amdgcn_exp2f((src[k * 2 * G + g] - mm) * LOG2E), ll);
    // a sequence with no live position at all (every position evicted by a forced plan) has m = -inf, l = 0 in every
    // split: its output is defined as zero, not 0/0
    M[t] = mm > -INFINITY ? mm : 0.f;
    IL[t] = ll > 0.f ? 1.0f / ll : 0.f;
  }
  __syncthreads();
  if (is_tile) {
    // 64 list entries per workgroup; thread (e, hg) sums the softmax weights of kv heads hg, hg+4, ... (all G members
    // of each), then the four partial sums of an entry are added in the fixed order hg = 0, 1, 2, 3
    const float pen = a.red ? a.red_w * (float)G / (float)(nF + nQ + nS) : 0.f;
    float acc = 0.f;
    if (pos >= 0) {
      for (int kvh = hg; kvh < a.Hkv; kvh += 4) {
        float x[G];
#pragma unroll
        for (int g = 0; g < G; ++g) x[g] = (kvh == hg) ? x0[g] : a.xs[((size_t)b * a.Hq + kvh * G + g) * a.xs_stride + j];
        if (a.vnorm) {
          // value-aware scorer: the group's weights times the norm of the value row its heads read
          float w = 0.f;
#pragma unroll
          for (int g = 0; g < G; ++g) w += __builtin_amdgcn_exp2f((x[g] - M[kvh * G + g]) * LOG2E) * IL[kvh * G + g];
          acc = fmaf(w, a.vnorm[((size_t)b * a.Hkv + kvh) * a.Nmax + pos], acc);
        } else {
#pragma unroll
          for (int g = 0; g < G; ++g) acc += __builtin_amdgcn_exp2f((x[g] - M[kvh * G + g]) * LOG2E) * IL[kvh * G + g];
        }
        // redundancy-penalised scorers: the G heads of the group each take red_w * rho / (positions attended) off
        if (a.red) acc = fmaf(-pen, a.red[((size_t)b * a.Hkv + kvh) * a.Nmax + pos], acc);
      }
    }
    __syncthreads();          // sm_pm is free now: reuse it for the partial sums
    sm_pm[hg * 64 + e] = acc;
    __syncthreads();
    if (hg == 0 && pos >= 0) {
      const float tot = ((sm_pm[e] + sm_pm[64 + e]) + sm_pm[128 + e]) + sm_pm[192 + e];
      a.score[(size_t)b * a.Nmax + pos] = score_old + a.score_scale * tot;
    }
  } else {
    // one workgroup per query head: thread (d, sg) sums the splits sg, sg+NSG, ... of output element d, then the NSG
    // partial sums are added in the fixed order sg = 0, 1, ...
    constexpr int NSG = 256 / D;
    const int hq = blockIdx.x - n_tiles, kvh = hq / G, h = hq % G;
    const int d = t % D, sg = t / D;
    const float* pm = in_lds ? (sm_pm + kvh * per_kvh) : (pmb + (size_t)kvh * a.S_total * 2 * G);
    const float* pob = a.part_o + ((size_t)(b * a.Hkv + kvh) * a.S_total * G) * D + h * D + d;
    const float mg = M[hq];
    float acc = 0.f;
#pragma unroll 8
    for (int k = sg; k < ns; k += NSG)
      acc = fmaf(__builtin_amdgcn_exp2f((pm[k * 2 * G + h] - mg) * LOG2E), pob[(size_t)k * G * D], acc);
    __syncthreads();          // every thread has read what it needs from sm_pm
    sm_pm[sg * D + d] = acc;
    __syncthreads();
    if (sg == 0) {
      float tot = sm_pm[d];
#pragma unroll
      for (int g2 = 1; g2 < NSG; ++g2) tot += sm_pm[g2 * D + d];
      tot *= IL[hq];
      const size_t oi = ((size_t)b * a.o_bs + hq) * D + d;
      if (a.out_kind == KT_BF16) ((uint16_t*)a.out)[oi] = f32_to_bf16(tot);
      else if (a.out_kind == KT_F16) ((_Float16*)a.out)[oi] = (_Float16)tot;    // round to nearest even
      else ((float*)a.out)[oi] = tot;
    }
  }
}

// ---- finish for several query tokens per sequence (one launch served n_q * cq of them) --------------------------
// Grid (64-entry slots of the last token's lists + Hq * queries, B).  Slot workgroups: every list entry gets the
// weights of the queries added in query order (what single-token calls would have done, with the same arithmetic per
// query: thread (e, hg) sums kv heads hg, hg+4, ..., the four partial sums are added in the order hg = 0..3).  Query
// jt does not see the last queries - 1 - jt entries of list F; its Q-list logits start where the F tiles of its
// group (the cq tokens of one workgroup, laid out for the group's last token) end.  The other workgroups merge the
// splits of one (query, head) into out.
template <int D, int G>
__global__ __launch_bounds__(256) void k_attn_finish_chunk(const AttnArgs a, int n_tiles) {
  constexpr int MAXQ = 16;
  __shared__ float M[MAXQ][128], IL[MAXQ][128];
  __shared__ float sm_part[4 * 256];
  const int t = threadIdx.x, b = blockIdx.y, nq = a.n_q * a.cq, ns = a.S_total;
  int nF, nQ;
  if (a.B <= ATTN_ARG_SEQS) { nF = a.nF[b]; nQ = a.nQ[b]; }
  else { nF = a.cnt[b * CNT_N + C_NF] - a.trim; nQ = a.cnt[b * CNT_N + C_NQ]; }
  const int cf = (nF + TB - 1) / TB;                       // F tiles of the last query (the longest list)
  const bool is_tile = (int)blockIdx.x < n_tiles;
  if (is_tile && (int)blockIdx.x * 64 >= cf * TB + nQ) return;
  // global (m, 1/l) of every (query, head) of this sequence
  for (int i = t; i < nq * a.Hq; i += 256) {
    const int jt = i / a.Hq, hq = i % a.Hq, kvh = hq / G, g = hq % G;
    const float* src = a.part_ml + (size_t)((b * nq + jt) * a.Hkv + kvh) * ns * 2 * G;
    float mm = -INFINITY;
    for (int k = 0; k < ns; ++k) mm = fmaxf(mm, src[k * 2 * G + g]);
    float ll = 0.f;
    for (int k = 0; k < ns; ++k) ll = fmaf(src[k * 2 * G + G + g], __builtin_amdgcn_exp2f((src[k * 2 * G + g] - mm) * LOG2E), ll);
    M[jt][hq] = mm > -INFINITY ? mm : 0.f;
    IL[jt][hq] = ll > 0.f ? 1.0f / ll : 0.f;
  }
  __syncthreads();
  if (is_tile) {
    const int e = t & 63, hg = t >> 6;
    const int sl = blockIdx.x * 64 + e;                     // slot in the last query's layout
    const bool is_f = sl < nF, is_q = sl >= cf * TB && sl - cf * TB < nQ;
    int pos = -1;
    if (is_f) pos = a.f_pos[(size_t)b * a.Nmax + sl];
    else if (is_q) pos = a.q_pos[(size_t)b * a.Nmax + (sl - cf * TB)];
    float score = (hg == 0 && pos >= 0) ? a.score[(size_t)b * a.Nmax + pos] : 0.f;
    // four tokens at a time: their sums are independent (all loads in flight together), only the additions into the
    // score go in token order
    for (int j0 = 0; j0 < nq; j0 += 4) {
      float acc[4];
      bool seen[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int jt = j0 + u;
        acc[u] = 0.f; seen[u] = false;
        if (jt >= nq) continue;
        const int nFj = nF - (nq - 1 - jt);                                   // what the query sees of list F
        const int cfz = (nF - (a.n_q - 1 - jt / a.cq) * a.cq + TB - 1) / TB;  // F tiles in its group's layout
        seen[u] = is_q || (is_f && sl < nFj);               // wave-divergent at most in a list's last tile
        const float pen = a.red ? a.red_w * (float)G / (float)(nFj + nQ) : 0.f;
        const int col = is_q ? cfz * TB + (sl - cf * TB) : sl;
        if (seen[u]) {
          for (int kvh = hg; kvh < a.Hkv; kvh += 4) {
            float x[G];
#pragma unroll
            for (int g = 0; g < G; ++g) x[g] = a.xs[((size_t)(b * nq + jt) * a.Hq + kvh * G + g) * a.xs_stride + col];
            if (a.vnorm) {
              float w = 0.f;
#pragma unroll
              for (int g = 0; g < G; ++g) w += __builtin_amdgcn_exp2f((x[g] - M[jt][kvh * G + g]) * LOG2E) * IL[jt][kvh * G + g];
              acc[u] = fmaf(w, a.vnorm[((size_t)b * a.Hkv + kvh) * a.Nmax + pos], acc[u]);
            } else {
#pragma unroll
              for (int g = 0; g < G; ++g) acc[u] += __builtin_amdgcn_exp2f((x[g] - M[jt][kvh * G + g]) * LOG2E) * IL[jt][kvh * G + g];
            }
            if (a.red) acc[u] = fmaf(-pen, a.red[((size_t)b * a.Hkv + kvh) * a.Nmax + pos], acc[u]);
          }
        }
      }
      __syncthreads();
#pragma unroll
      for (int u = 0; u < 4; ++u) sm_part[u * 256 + hg * 64 + e] = acc[u];
      __syncthreads();
      if (hg == 0) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (seen[u]) score = score + a.score_scale * (((sm_part[u * 256 + e] + sm_part[u * 256 + 64 + e]) + sm_part[u * 256 + 128 + e]) + sm_part[u * 256 + 192 + e]);
      }
    }
    if (hg == 0 && pos >= 0) a.score[(size_t)b * a.Nmax + pos] = score;
  } else {
    constexpr int NSG = 256 / D;
    const int idx = blockIdx.x - n_tiles, jt = idx / a.Hq, hq = idx % a.Hq, kvh = hq / G, h = hq % G;
    const int d = t % D, sg = t / D;
    const float* pm = a.part_ml + (size_t)((b * nq + jt) * a.Hkv + kvh) * ns * 2 * G;
    const float* pob = a.part_o + ((size_t)((b * nq + jt) * a.Hkv + kvh) * ns * G) * D + h * D + d;
    const float mg = M[jt][hq];
    float acc = 0.f;
#pragma unroll 4
    for (int k = sg; k < ns; k += NSG)
      acc = fmaf(__builtin_amdgcn_exp2f((pm[k * 2 * G + h] - mg) * LOG2E), pob[(size_t)k * G * D], acc);
    sm_part[sg * D + d] = acc;
    __syncthreads();
    if (sg == 0) {
      float tot = sm_part[d];
#pragma unroll
      for (int g2 = 1; g2 < NSG; ++g2) tot += sm_part[g2 * D + d];
      tot *= IL[jt][hq];
      const size_t oi = ((size_t)b * a.o_bs + (size_t)jt * a.Hq + hq) * D + d;
      if (a.out_kind == KT_BF16) ((uint16_t*)a.out)[oi] = f32_to_bf16(tot);
      else if (a.out_kind == KT_F16) ((_Float16*)a.out)[oi] = (_Float16)tot;
      else ((float*)a.out)[oi] = tot;
    }
  }
}

// ---- dispatch ----------------------------------------------------------------------------------------------
// The file is compiled once per part (TKV_ATTN_PART = 0..3, 5, 6: one (head_dim, KV dtype) pair of attn_tiered each,
// 4: attn_finish and the launchers), so the parts build in parallel; without the macro it is one translation unit.
#if defined(TKV_ATTN_PART)
#define TKV_HAS_PART(p) (TKV_ATTN_PART == (p))
#else
#define TKV_HAS_PART(p) 1
#endif

#define TKV_DISPATCH_G(FN, D_, BF_, ...)                    \
  switch (G) {                                              \
    case 1: return FN<D_, 1, BF_>(__VA_ARGS__);             \
    case 2: return FN<D_, 2, BF_>(__VA_ARGS__);             \
    case 3: return FN<D_, 3, BF_>(__VA_ARGS__);             \
    case 4: return FN<D_, 4, BF_>(__VA_ARGS__);             \
    case 5: return FN<D_, 5, BF_>(__VA_ARGS__);             \
    case 6: return FN<D_, 6, BF_>(__VA_ARGS__);             \
    case 7: return FN<D_, 7, BF_>(__VA_ARGS__);             \
    case 8: return FN<D_, 8, BF_>(__VA_ARGS__);             \
    default: return hipErrorInvalidValue;                   \
  }

// With a pair of events the launch is timed by the dispatch's own begin / end timestamps (no bracket overhead).
template <int D, int G, int KT>
static hipError_t run_tiered(const AttnArgs& a, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  dim3 grid(a.S, a.Hkv, a.B * a.n_q);
  // One query token per workgroup (a decode step; binary32 rows always): the vector kernel, G dot products per row.
  // Several query tokens as columns of one workgroup (16-bit rows): a (rows x D) by (D x G * cq) contraction, on the
  // matrix cores.
  if (a.cq == 1) {
    constexpr int threads = KernelGeo<D, G, KT>::NW * 64;
    if (ev0 && ev1) hipExtLaunchKernelGGL((k_attn_tiered<D, G, KT>), grid, dim3(threads), 0, st, ev0, ev1, 0, a);
    else hipLaunchKernelGGL((k_attn_tiered<D, G, KT>), grid, dim3(threads), 0, st, a);
  } else if constexpr (KT == KT_F32) {
    return hipErrorInvalidValue;
  } else {
    if (a.cq < 1 || a.cq * G > 32) return hipErrorInvalidValue;
    if (a.cq * G <= 16) {
      if (ev0 && ev1) hipExtLaunchKernelGGL((k_attn_tiered_mc<D, G, KT, 1>), grid, dim3(mc_waves(1) * 64), 0, st, ev0, ev1, 0, a);
      else hipLaunchKernelGGL((k_attn_tiered_mc<D, G, KT, 1>), grid, dim3(mc_waves(1) * 64), 0, st, a);
    } else {
      if (ev0 && ev1) hipExtLaunchKernelGGL((k_attn_tiered_mc<D, G, KT, 2>), grid, dim3(mc_waves(2) * 64), 0, st, ev0, ev1, 0, a);
      else hipLaunchKernelGGL((k_attn_tiered_mc<D, G, KT, 2>), grid, dim3(mc_waves(2) * 64), 0, st, a);
    }
  }
  return hipGetLastError();
}
template <int D, int KT>
hipError_t tiered_by_group(const AttnArgs& a, int G, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1);
#define TKV_DEFINE_PART(D_, BF_)                                                                                   \
  template <>                                                                                                      \
  hipError_t tiered_by_group<D_, BF_>(const AttnArgs& a, int G, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {  \
    TKV_DISPATCH_G(run_tiered, D_, BF_, a, st, ev0, ev1)                                                           \
  }
#if TKV_HAS_PART(0)
TKV_DEFINE_PART(128, KT_BF16)
#endif
#if TKV_HAS_PART(1)
TKV_DEFINE_PART(128, KT_F32)
#endif
#if TKV_HAS_PART(2)
TKV_DEFINE_PART(64, KT_BF16)
#endif
#if TKV_HAS_PART(3)
TKV_DEFINE_PART(64, KT_F32)
#endif
#if TKV_HAS_PART(5)
TKV_DEFINE_PART(128, KT_F16)
#endif
#if TKV_HAS_PART(6)
TKV_DEFINE_PART(64, KT_F16)
#endif

#if TKV_HAS_PART(4)
template <> hipError_t tiered_by_group<128, KT_BF16>(const AttnArgs&, int, hipStream_t, hipEvent_t, hipEvent_t);
template <> hipError_t tiered_by_group<128, KT_F32>(const AttnArgs&, int, hipStream_t, hipEvent_t, hipEvent_t);
template <> hipError_t tiered_by_group<128, KT_F16>(const AttnArgs&, int, hipStream_t, hipEvent_t, hipEvent_t);
template <> hipError_t tiered_by_group<64, KT_BF16>(const AttnArgs&, int, hipStream_t, hipEvent_t, hipEvent_t);
template <> hipError_t tiered_by_group<64, KT_F32>(const AttnArgs&, int, hipStream_t, hipEvent_t, hipEvent_t);
template <> hipError_t tiered_by_group<64, KT_F16>(const AttnArgs&, int, hipStream_t, hipEvent_t, hipEvent_t);

template <int D, int G, int KT>
static hipError_t run_finish(const AttnArgs& a, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  const int tiles = a.n_tiles;
  if (ev0 && ev1) hipExtLaunchKernelGGL((k_attn_finish<D, G>), dim3(tiles + a.Hq, a.B), dim3(256), 0, st, ev0, ev1, 0, a, tiles);
  else hipLaunchKernelGGL((k_attn_finish<D, G>), dim3(tiles + a.Hq, a.B), dim3(256), 0, st, a, tiles);
  return hipGetLastError();
}

hipError_t launch_attn_tiered(const AttnArgs& a, int D, int G, int kt, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  if (D == 128 && kt == KT_BF16) return tiered_by_group<128, KT_BF16>(a, G, st, ev0, ev1);
  if (D == 128 && kt == KT_F32) return tiered_by_group<128, KT_F32>(a, G, st, ev0, ev1);
  if (D == 128 && kt == KT_F16) return tiered_by_group<128, KT_F16>(a, G, st, ev0, ev1);
  if (D == 64 && kt == KT_BF16) return tiered_by_group<64, KT_BF16>(a, G, st, ev0, ev1);
  if (D == 64 && kt == KT_F32) return tiered_by_group<64, KT_F32>(a, G, st, ev0, ev1);
  if (D == 64 && kt == KT_F16) return tiered_by_group<64, KT_F16>(a, G, st, ev0, ev1);
  return hipErrorInvalidValue;
}
int attn_waves_per_group(int D, int elem_bytes, int G, int cq) {
  return (elem_bytes == 2 && cq > 1) ? mc_waves(cq * G <= 16 ? 1 : 2) : waves_per_group(D * elem_bytes, G);
}
int attn_cols_per_launch(int elem_bytes, int G) { return elem_bytes == 2 ? (32 / G < 16 ? 32 / G : 16) : 1; }
int attn_q_waves(int n_waves, int n_f_tiles, int n_q_tiles) { return q_waves(n_waves, n_f_tiles, n_q_tiles); }

template <int D, int G, int KT>
static hipError_t run_finish_chunk(const AttnArgs& a, hipStream_t st) {
  hipLaunchKernelGGL((k_attn_finish_chunk<D, G>), dim3(a.n_tiles + a.Hq * a.n_q * a.cq, a.B), dim3(256), 0, st, a, a.n_tiles);
  return hipGetLastError();
}
hipError_t launch_attn_finish_chunk(const AttnArgs& a, int D, int G, hipStream_t st) {
  if (a.n_q < 1 || a.cq < 1 || a.n_q * a.cq > 16 || a.Hq > 128) return hipErrorInvalidValue;
  if (D == 128) { TKV_DISPATCH_G(run_finish_chunk, 128, KT_BF16, a, st) }
  if (D == 64) { TKV_DISPATCH_G(run_finish_chunk, 64, KT_BF16, a, st) }
  return hipErrorInvalidValue;
}

hipError_t launch_attn_finish(const AttnArgs& a, int D, int G, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  if (D == 128) { TKV_DISPATCH_G(run_finish, 128, KT_BF16, a, st, ev0, ev1) }
  if (D == 64) { TKV_DISPATCH_G(run_finish, 64, KT_BF16, a, st, ev0, ev1) }
  return hipErrorInvalidValue;
}

// ---- bandwidth probe: what a plain streaming read of `bytes` reaches with the attention kernel's launch shape ----
// One workgroup per compute unit, 512 lanes, 16-byte loads, four independent loads in flight per lane; nothing is
// written unless the data says so (it never does for the probe's buffer), so the traffic is the read alone.
__global__ __launch_bounds__(512) void k_probe_read(const u32x4* __restrict__ src, size_t n16, uint32_t* sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t acc = 0;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride);
    const u32x4 c = __builtin_nontemporal_load(src + i + 2 * stride), d = __builtin_nontemporal_load(src + i + 3 * stride);
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < n16; i += stride) { const u32x4 a = __builtin_nontemporal_load(src + i); acc ^= a.x ^ a.y ^ a.z ^ a.w; }
  if (acc == 0x9E3779B9u) *sink = acc;
}
hipError_t launch_probe_read(const void* src, size_t bytes, int workgroups, uint32_t* sink, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  hipExtLaunchKernelGGL(k_probe_read, dim3(workgroups), dim3(512), 0, st, ev0, ev1, 0, (const u32x4*)src, bytes / 16, sink);
  return hipGetLastError();
}
#endif

}  // namespace tkv
