// Decode attention over the tiered KV cache, with cumulative-score emission (Eq. 1, Eq. 2-3 of the paper).
//
//   attn_tiered : grid (S, Hkv, B), 4 waves per workgroup.  Workgroup (s, kvh, b) owns TOK_PER_BLOCK consecutive
//                 entries of one of the two per-sequence lists -- F (T0 u T1 rows at full precision, ascending
//                 position) or Q (T2 rows, int8 / int4 codes dequantised in registers); T3 positions are in
//                 neither list.  Every wave is autonomous and works on 64-entry tiles:
//                   K rows  - 8 lanes per row (each lane 1/8 of the row), 8 rows per wave-wide load; the G logits
//                             of a row are reduced over its 8 lanes by DPP and kept by the lane whose index
//                             equals the entry's index in the tile, so after 8 loads lane i holds entry i;
//                   softmax - online, one entry per lane (exact tile maximum, exp2, running m and l);
//                   V rows  - 16 bytes per lane, 64/LPR rows per wave-wide load, probabilities broadcast from
//                             LDS, per-lane fp32 output slices.
//                 The four waves are merged through LDS into one split partial (m, l, o[G][D]); the scaled
//                 logits go to a scratch array.
//   attn_finish : grid (64-entry tiles + Hq, B).  Every workgroup first merges the (m, l) of all splits of its sequence
//                 into the global (m, 1/l) of every query head.  Tile workgroups then turn the stored logits
//                 into softmax weights, summed over all query heads in a fixed order, into score[b, pos]; the
//                 Hq remaining workgroups merge the split outputs of one query head each into out[b, hq].
// The split boundaries and the fp32 summation order depend only on the lists' logical order, never on whether a
// row lives in the HBM pool or the staging buffer (both are one slot space), which is what makes T1 placement
// bit-invisible (Prop. 1).  No MFMA: the path is bound by HBM, and the per-row work is G dot products.
#include <hip/hip_ext.h>

#include "tkv_internal.h"

namespace tkv {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

constexpr float LOG2E = 1.4426950408889634f;
constexpr int TB = TOK_PER_BLOCK;
constexpr int NWAVE = ATTN_THREADS / 64;
constexpr int TPW = TB / NWAVE;   // list entries per wave
constexpr int NTILE = TPW / 64;   // 64-entry tiles per wave
static_assert(TPW % 64 == 0 && NTILE >= 1, "a wave works in tiles of 64 entries");

#ifndef TKV_UK
#define TKV_UK 2      // K rows per batch and lane group (two batches are in flight)
#endif
#ifndef TKV_UV
#define TKV_UV 4      // V rows per batch and lane group (two batches are in flight)
#endif
#ifndef TKV_DEEP
#define TKV_DEEP 0
#endif
#ifdef TKV_ATTN_WAVES_PER_EU
#define TKV_WPE __attribute__((amdgpu_waves_per_eu(TKV_ATTN_WAVES_PER_EU, TKV_ATTN_WAVES_PER_EU)))
#else
#define TKV_WPE
#endif

enum Mode : int { F_BF16 = 0, F_F32 = 1, Q_INT8 = 2, Q_INT4 = 3 };

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
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
  if constexpr (LPR >= 32) x += __shfl_xor(x, 16);
  return x;
}
__device__ __forceinline__ float rdlane(float x, int l) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), l));
}

// whole-wave reductions: 16-lane rows by DPP, rows 0/1 and 2/3 by row_bcast15, halves by row_bcast31; lane 63 has
// the result, which is returned in a scalar register
__device__ __forceinline__ float wave_max(float x) {
  x = fmaxf(x, dpp_f<0xB1>(x)); x = fmaxf(x, dpp_f<0x4E>(x)); x = fmaxf(x, dpp_f<0x141>(x)); x = fmaxf(x, dpp_f<0x140>(x));
  x = fmaxf(x, dpp_rows<0x142, 0xA>(x));
  x = fmaxf(x, dpp_rows<0x143, 0xC>(x));
  return rdlane(x, 63);
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
// two code values (exact in bf16: at most 8 significant bits) packed as a bf16 pair
__device__ __forceinline__ uint32_t pack_bf16_pair(float lo, float hi) {
  return (__builtin_bit_cast(uint32_t, hi) & 0xffff0000u) | (__builtin_bit_cast(uint32_t, lo) >> 16);
}

template <int G>
struct GPad { static constexpr int v = (G <= 4) ? 4 : 8; };

// ---- geometry ------------------------------------------------------------------------------------------------
template <int D, Mode M>
struct Geo {
  static constexpr bool IS_Q = (M == Q_INT8 || M == Q_INT4);
  // K side: 8 lanes per row
  static constexpr int EK = D / 8;                                            // elements of a K row per lane
  static constexpr int KDW = (M == F_BF16) ? EK / 2 : (M == F_F32) ? EK : (M == Q_INT8) ? EK / 4 : EK / 8;  // dwords per lane
  // V side: one 16-byte piece (F modes) / 8 codes (Q modes) per lane
  static constexpr int EV = (M == F_F32) ? 4 : 8;
  static constexpr int LPRV = D / EV;                                         // lanes per V row
  static constexpr int NITV = LPRV;                                           // wave-wide V loads per tile
  static constexpr float OFF = (M == Q_INT4) ? 8.f : 128.f;                   // codes are read as code + OFF
};

struct RowSrc {
  __amdgpu_buffer_rsrc_t data, scale;
  uint32_t row_bytes, scale_bytes;
};

template <int NDW>
__device__ __forceinline__ void load_dwords(const __amdgpu_buffer_rsrc_t& rs, uint32_t off, uint32_t (&w)[NDW]) {
  if constexpr (NDW >= 4) {
#pragma unroll
    for (int i = 0; i < NDW / 4; ++i) {
      const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, off + 16 * i, 0, 2);
      w[4 * i] = v.x; w[4 * i + 1] = v.y; w[4 * i + 2] = v.z; w[4 * i + 3] = v.w;
    }
  } else if constexpr (NDW == 2) {
    const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rs, off, 0, 2);
    w[0] = v.x; w[1] = v.y;
  } else {
    w[0] = __builtin_amdgcn_raw_buffer_load_b32(rs, off, 0, 2);
  }
}

// scale of a T2 row (INT8) or of the 32-code group that starts at element e0 (INT4).  loc == -1 is out of range: 0
template <Mode M>
__device__ __forceinline__ float load_scale(const RowSrc& s, int loc, int e0) {
  if constexpr (M == Q_INT8) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(s.scale, (uint32_t)loc * s.scale_bytes, 0, 0));
  } else if constexpr (M == Q_INT4) {
    const uint16_t hb = __builtin_amdgcn_raw_buffer_load_b16(s.scale, (uint32_t)loc * s.scale_bytes + (uint32_t)(e0 >> 5) * 2, 0, 0);
    return (float)__builtin_bit_cast(_Float16, hb);
  } else {
    return 0.f;
  }
}

template <int D, Mode M>
struct KRow { uint32_t w[Geo<D, M>::KDW]; float sc; };
template <int D, Mode M>
struct VRow { uint32_t w[(M == Q_INT8) ? 2 : (M == Q_INT4) ? 1 : 4]; float sc; };

// loc == -1 gives offsets beyond the buffer: such loads return zeros
template <int D, Mode M>
__device__ __forceinline__ KRow<D, M> load_krow(const RowSrc& s, int loc, int r8) {
  KRow<D, M> out;
  load_dwords<Geo<D, M>::KDW>(s.data, (uint32_t)loc * s.row_bytes + (uint32_t)r8 * (Geo<D, M>::KDW * 4), out.w);
  out.sc = load_scale<M>(s, loc, r8 * Geo<D, M>::EK);
  return out;
}
template <int D, Mode M>
__device__ __forceinline__ VRow<D, M> load_vrow(const RowSrc& s, int loc, int r) {
  VRow<D, M> out;
  constexpr int NDW = (M == Q_INT8) ? 2 : (M == Q_INT4) ? 1 : 4;
  load_dwords<NDW>(s.data, (uint32_t)loc * s.row_bytes + (uint32_t)r * (NDW * 4), out.w);
  out.sc = load_scale<M>(s, loc, r * 8);
  return out;
}

// codes as unsigned values code + OFF; the offset is removed once per row: sum q*(u-OFF) = sum q*u - OFF*sum q
template <Mode M, int NDW>
__device__ __forceinline__ void unpack_codes(const uint32_t (&w)[NDW], float (&f)[(M == Q_INT8) ? NDW * 4 : NDW * 8]) {
  if constexpr (M == Q_INT8) {
#pragma unroll
    for (int i = 0; i < NDW; ++i) {
      const uint32_t u = w[i] ^ 0x80808080u;
#pragma unroll
      for (int n = 0; n < 4; ++n) f[i * 4 + n] = (float)((u >> (8 * n)) & 0xFFu);
    }
  } else {
#pragma unroll
    for (int i = 0; i < NDW; ++i) {
      const uint32_t u = w[i] ^ 0x88888888u;
#pragma unroll
      for (int n = 0; n < 8; ++n) f[i * 8 + n] = (float)((u >> (4 * n)) & 0xFu);
    }
  }
}

// The lane's 1/8 slice of the G query vectors.  bf16 queries stay packed (EK/2 dwords per head, fed to the bf16
// dot instruction); binary32 queries are kept as EK floats.  qs is the slice's sum (Q modes only).
template <int D, int G, bool QBF>
struct QRegs {
  static constexpr int EK = D / 8;
  uint32_t qp[QBF ? G : 1][EK / 2];
  float qf[QBF ? 1 : G][EK];
  float qs[G];
};

// G logits of one K row, reduced over the row's 8 lanes (every lane of the group gets them)
template <int D, int G, Mode M, bool QBF>
__device__ __forceinline__ void row_logits(const KRow<D, M>& kr, const QRegs<D, G, QBF>& q, float (&x)[G]) {
  using GE = Geo<D, M>;
  constexpr int EK = GE::EK;
  if constexpr (M == F_BF16) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float acc = 0.f;
#pragma unroll
      for (int c = 0; c < EK / 2; ++c)
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, kr.w[c]), __builtin_bit_cast(bf16x2, q.qp[h][c]), acc, false);
      x[h] = group_sum<8>(acc);
    }
  } else if constexpr (M == F_F32) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float acc = 0.f;
#pragma unroll
      for (int c = 0; c < EK; ++c) acc = fmaf(__builtin_bit_cast(float, kr.w[c]), q.qf[h][c], acc);
      x[h] = group_sum<8>(acc);
    }
  } else {
    float kf[EK];
    unpack_codes<M, GE::KDW>(kr.w, kf);
    uint32_t kp[EK / 2];
    if constexpr (QBF) {
#pragma unroll
      for (int c = 0; c < EK / 2; ++c) kp[c] = pack_bf16_pair(kf[2 * c], kf[2 * c + 1]);
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float acc = -GE::OFF * q.qs[h];
      if constexpr (QBF) {
#pragma unroll
        for (int c = 0; c < EK / 2; ++c)
          acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, kp[c]), __builtin_bit_cast(bf16x2, q.qp[h][c]), acc, false);
      } else {
#pragma unroll
        for (int c = 0; c < EK; ++c) acc = fmaf(q.qf[h][c], kf[c], acc);
      }
      if constexpr (M == Q_INT4) acc *= kr.sc;      // per-group scale: before the cross-lane sum
      x[h] = group_sum<8>(acc);
      if constexpr (M == Q_INT8) x[h] *= kr.sc;     // per-row scale
    }
  }
}

template <int D, int G, Mode M>
__device__ __forceinline__ void row_accumulate(const VRow<D, M>& vr, const float (&p)[GPad<G>::v],
                                               float (&o)[G][Geo<D, M>::EV], float (&osub)[G]) {
  constexpr int EV = Geo<D, M>::EV;
  if constexpr (M == F_BF16) {
    float vf[8];
#pragma unroll
    for (int c = 0; c < 4; ++c) { vf[2 * c] = bf_lo(vr.w[c]); vf[2 * c + 1] = bf_hi(vr.w[c]); }
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < EV; ++e) o[h][e] = fmaf(p[h], vf[e], o[h][e]);
  } else if constexpr (M == F_F32) {
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < EV; ++e) o[h][e] = fmaf(p[h], __builtin_bit_cast(float, vr.w[e]), o[h][e]);
  } else {
    float vf[8];
    unpack_codes<M, (M == Q_INT8) ? 2 : 1>(vr.w, vf);
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float ps = p[h] * vr.sc;
      osub[h] += ps;
#pragma unroll
      for (int e = 0; e < EV; ++e) o[h][e] = fmaf(ps, vf[e], o[h][e]);
    }
  }
}

// ---- one workgroup: TOK_PER_BLOCK entries of list F or Q --------------------------------------------------
// Leaves the workgroup's split partial in part_ml / part_o and the scaled logits in xs.
template <int D, int G, Mode M, bool QBF>
__device__ __forceinline__ void attn_block(const AttnArgs& a, float* sm_o, float* sm_ml, float* pbuf_all,
                                           int b, int kvh, int s, int ntok, const int* loc_list) {
  using GE = Geo<D, M>;
  constexpr int EV = GE::EV, LPRV = GE::LPRV, NITV = GE::NITV, EK = GE::EK;
  constexpr int GP = GPad<G>::v;
  constexpr int UK = TKV_UK, NBK = 8 / UK;            // K: 8 wave-wide loads per tile, in batches of UK
  constexpr int UV = (TKV_UV * 2 <= NITV) ? TKV_UV : NITV / 2, NBV = NITV / UV;   // V: NITV loads per tile
  static_assert(NITV % UV == 0 && NBV % 2 == 0 && NBK % 2 == 0, "batches come in pairs");
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int g8 = lane >> 3, r8 = lane & 7;           // K side: row group and slice
  const int gv = lane / LPRV, rv = lane % LPRV;      // V side
  float* pbuf = pbuf_all + wave * 64 * GP;

  RowSrc ks, vs;
  if constexpr (!GE::IS_Q) {
    const uint32_t rb = D * (QBF ? 2u : 4u);
    const size_t off = (size_t)(b * a.Hkv + kvh) * a.capF * rb;
    ks.data = make_rsrc(a.fpK + off, (uint32_t)a.capF * rb); vs.data = make_rsrc(a.fpV + off, (uint32_t)a.capF * rb);
    ks.scale = ks.data; vs.scale = vs.data;
    ks.row_bytes = vs.row_bytes = rb; ks.scale_bytes = vs.scale_bytes = 0;
  } else {
    const size_t rows = (size_t)(b * a.Hkv + kvh) * a.cap2;
    ks.data = make_rsrc(a.c2K + rows * a.cb, (uint32_t)a.cap2 * a.cb); vs.data = make_rsrc(a.c2V + rows * a.cb, (uint32_t)a.cap2 * a.cb);
    ks.scale = make_rsrc(a.s2K + rows * a.sb, (uint32_t)a.cap2 * a.sb); vs.scale = make_rsrc(a.s2V + rows * a.sb, (uint32_t)a.cap2 * a.sb);
    ks.row_bytes = vs.row_bytes = a.cb; ks.scale_bytes = vs.scale_bytes = a.sb;
  }

  // this lane's 1/8 slice of the G query vectors
  QRegs<D, G, QBF> q;
  {
    constexpr int qes = QBF ? 2 : 4;
    const char* qb = (const char*)a.q + ((size_t)(b * a.Hq + kvh * G) * D + r8 * EK) * qes;
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const char* qh = qb + (size_t)h * D * qes;
      float sacc = 0.f;
      if constexpr (QBF) {
#pragma unroll
        for (int c = 0; c < EK / 8; ++c) {
          const u32x4 v = *(const u32x4*)(qh + 16 * c);
          q.qp[h][4 * c] = v.x; q.qp[h][4 * c + 1] = v.y; q.qp[h][4 * c + 2] = v.z; q.qp[h][4 * c + 3] = v.w;
        }
        if constexpr (GE::IS_Q) {
#pragma unroll
          for (int c = 0; c < EK / 2; ++c) sacc += bf_lo(q.qp[h][c]) + bf_hi(q.qp[h][c]);
        }
      } else {
#pragma unroll
        for (int c = 0; c < EK / 4; ++c) {
          const float4 v = *(const float4*)(qh + 16 * c);
          q.qf[h][4 * c] = v.x; q.qf[h][4 * c + 1] = v.y; q.qf[h][4 * c + 2] = v.z; q.qf[h][4 * c + 3] = v.w;
        }
        if constexpr (GE::IS_Q) {
#pragma unroll
          for (int c = 0; c < EK; ++c) sacc += q.qf[h][c];
        }
      }
      q.qs[h] = sacc;
    }
  }

  float o[G][EV], osub[G], m_run[G], l_run[G];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    osub[h] = 0.f; m_run[h] = -INFINITY; l_run[h] = 0.f;
#pragma unroll
    for (int e = 0; e < EV; ++e) o[h][e] = 0.f;
  }

  // Two schedules for the tile loop.  DEEP keeps a whole tile's K rows and V rows in flight (128 registers of
  // buffers, two waves per SIMD) and fetches the next tile's rows while the current one is being computed; the
  // batched schedule keeps two small batches in flight and fits three or four waves per SIMD.
  constexpr bool DEEP = (TKV_DEEP != 0) && (G <= 6) && (M != F_F32);
  if constexpr (DEEP) {
    KRow<D, M> kb[8];
    VRow<D, M> vb[NITV];
    int locs[NTILE];
#pragma unroll
    for (int tl = 0; tl < NTILE; ++tl) {
      const int tb2 = wave * TPW + tl * 64;
      locs[tl] = (tb2 + lane < ntok) ? loc_list[tb2 + lane] : -1;
    }
    auto issue_k_all = [&](int myloc) {
#pragma unroll
      for (int it = 0; it < 8; ++it) kb[it] = load_krow<D, M>(ks, __shfl(myloc, g8 * 8 + it), r8);
    };
    auto issue_v_all = [&](int myloc) {
#pragma unroll
      for (int it = 0; it < NITV; ++it) vb[it] = load_vrow<D, M>(vs, __shfl(myloc, gv * LPRV + it), rv);
    };
    issue_k_all(locs[0]);
    issue_v_all(locs[0]);
#pragma unroll
    for (int tile = 0; tile < NTILE; ++tile) {
      const int tbase = wave * TPW + tile * 64;
      if (tbase >= ntok) break;                          // wave-uniform
      const bool valid = tbase + lane < ntok;
      float xt[G];
#pragma unroll
      for (int h = 0; h < G; ++h) xt[h] = 0.f;
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        float x[G];
        row_logits<D, G, M, QBF>(kb[it], q, x);
#pragma unroll
        for (int h = 0; h < G; ++h) xt[h] = (r8 == it) ? x[h] : xt[h];
        __builtin_amdgcn_sched_barrier(0);
      }
      if (tile + 1 < NTILE) issue_k_all(locs[tile + 1 < NTILE ? tile + 1 : tile]);   // out-of-range slots cost nothing
      float corr[G];
      {
        const size_t xbase = ((size_t)(b * a.Hq + kvh * G)) * a.xs_stride + (size_t)s * TB + tbase + lane;
#pragma unroll
        for (int h = 0; h < G; ++h) {
          const float x = valid ? xt[h] * a.softmax_scale : -INFINITY;
          if (valid) a.xs[xbase + (size_t)h * a.xs_stride] = x;
          const float tm = wave_max(x);
          float mn;
          if (tile == 0) { mn = tm; corr[h] = 0.f; }
          else { mn = fmaxf(m_run[h], tm); corr[h] = __builtin_amdgcn_exp2f((m_run[h] - mn) * LOG2E); }
          const float p = valid ? __builtin_amdgcn_exp2f((x - mn) * LOG2E) : 0.f;
          const float ps = wave_sum(p);
          l_run[h] = (tile == 0) ? ps : fmaf(l_run[h], corr[h], ps);
          m_run[h] = mn;
          pbuf[lane * GP + h] = p;
        }
      }
      __builtin_amdgcn_wave_barrier();
      if (tile > 0) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
          osub[h] *= corr[h];
#pragma unroll
          for (int e = 0; e < EV; ++e) o[h][e] *= corr[h];
        }
      }
#pragma unroll
      for (int it = 0; it < NITV; ++it) {
        float p[GP];
#pragma unroll
        for (int c = 0; c < GP; c += 4) {
          const float4 pv = *(const float4*)(pbuf + (gv * LPRV + it) * GP + c);
          p[c] = pv.x; p[c + 1] = pv.y; p[c + 2] = pv.z; p[c + 3] = pv.w;
        }
        row_accumulate<D, G, M>(vb[it], p, o, osub);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (tile + 1 < NTILE) issue_v_all(locs[tile + 1 < NTILE ? tile + 1 : tile]);
      __builtin_amdgcn_wave_barrier();
    }
  } else {
#pragma unroll
  for (int tile = 0; tile < NTILE; ++tile) {
    const int tbase = wave * TPW + tile * 64;          // first entry of the tile, relative to the workgroup
    if (tbase >= ntok) break;                          // wave-uniform
    const bool valid = tbase + lane < ntok;
    const int myloc = valid ? loc_list[tbase + lane] : -1;   // slot of tile entry `lane`

    // ---- K rows: entry g8*8 + it is loaded by lane group g8 at iteration it, two batches in flight
    KRow<D, M> kb0[UK], kb1[UK];
    auto issue_k = [&](int batch, KRow<D, M> (&dst)[UK]) {
#pragma unroll
      for (int u = 0; u < UK; ++u) dst[u] = load_krow<D, M>(ks, __shfl(myloc, g8 * 8 + batch * UK + u), r8);
    };
    float xt[G];
#pragma unroll
    for (int h = 0; h < G; ++h) xt[h] = 0.f;
    auto logits = [&](int batch, const KRow<D, M> (&src)[UK]) {
#pragma unroll
      for (int u = 0; u < UK; ++u) {
        float x[G];
        row_logits<D, G, M, QBF>(src[u], q, x);
        const int it = batch * UK + u;
#pragma unroll
        for (int h = 0; h < G; ++h) xt[h] = (r8 == it) ? x[h] : xt[h];   // lane g8*8+it keeps entry g8*8+it
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    issue_k(0, kb0);
    issue_k(1, kb1);
#pragma unroll 1
    for (int k = 0; k < NBK; k += 2) {
      logits(k, kb0);
      if (k + 2 < NBK) issue_k(k + 2, kb0);
      logits(k + 1, kb1);
      if (k + 3 < NBK) issue_k(k + 3, kb1);
    }
    // ---- V rows: entry gv*LPRV + it is loaded by lane group gv at iteration it; the first two batches fly
    //      while the softmax is computed
    VRow<D, M> vb0[UV], vb1[UV];
    auto issue_v = [&](int batch, VRow<D, M> (&dst)[UV]) {
#pragma unroll
      for (int u = 0; u < UV; ++u) dst[u] = load_vrow<D, M>(vs, __shfl(myloc, gv * LPRV + batch * UV + u), rv);
    };
    issue_v(0, vb0);
    issue_v(1, vb1);
    // ---- online softmax, one entry per lane
    float corr[G];
    {
      const size_t xbase = ((size_t)(b * a.Hq + kvh * G)) * a.xs_stride + (size_t)s * TB + tbase + lane;
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float x = valid ? xt[h] * a.softmax_scale : -INFINITY;
        if (valid) a.xs[xbase + (size_t)h * a.xs_stride] = x;
        const float tm = wave_max(x);
        float mn;
        if (tile == 0) { mn = tm; corr[h] = 0.f; }
        else { mn = fmaxf(m_run[h], tm); corr[h] = __builtin_amdgcn_exp2f((m_run[h] - mn) * LOG2E); }
        const float p = valid ? __builtin_amdgcn_exp2f((x - mn) * LOG2E) : 0.f;
        const float ps = wave_sum(p);
        l_run[h] = (tile == 0) ? ps : fmaf(l_run[h], corr[h], ps);
        m_run[h] = mn;
        pbuf[lane * GP + h] = p;
      }
    }
    __builtin_amdgcn_wave_barrier();
    if (tile > 0) {
#pragma unroll
      for (int h = 0; h < G; ++h) {
        osub[h] *= corr[h];
#pragma unroll
        for (int e = 0; e < EV; ++e) o[h][e] *= corr[h];
      }
    }
    // probabilities of entry (gv, it): read one row ahead of their use, so only two rows' worth stay in registers
    auto load_p = [&](int it, float (&p)[GP]) {
#pragma unroll
      for (int c = 0; c < GP; c += 4) {
        const float4 pv = *(const float4*)(pbuf + (gv * LPRV + it) * GP + c);
        p[c] = pv.x; p[c + 1] = pv.y; p[c + 2] = pv.z; p[c + 3] = pv.w;
      }
    };
    auto accum = [&](int batch, const VRow<D, M> (&src)[UV]) {
      float pc[GP];
      load_p(batch * UV, pc);
#pragma unroll
      for (int u = 0; u < UV; ++u) {
        float pn[GP];
        if (u + 1 < UV) load_p(batch * UV + u + 1, pn);
        __builtin_amdgcn_sched_barrier(0);   // rows stay in order: bounds the live p / widened-V registers
        row_accumulate<D, G, M>(src[u], pc, o, osub);
        __builtin_amdgcn_sched_barrier(0);
        if (u + 1 < UV) {
#pragma unroll
          for (int c = 0; c < GP; ++c) pc[c] = pn[c];
        }
      }
    };
#pragma unroll 1
    for (int k = 0; k < NBV; k += 2) {
      accum(k, vb0);
      if (k + 2 < NBV) issue_v(k + 2, vb0);
      accum(k + 1, vb1);
      if (k + 3 < NBV) issue_v(k + 3, vb1);
    }
    __builtin_amdgcn_wave_barrier();
  }
  }
  if constexpr (GE::IS_Q) {
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < EV; ++e) o[h][e] = fmaf(-GE::OFF, osub[h], o[h][e]);
  }
  // ---- wave partial: sum the row groups, then merge the four waves through LDS
#pragma unroll
  for (int st = LPRV; st < 64; st <<= 1) {
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < EV; ++e) o[h][e] += __shfl_xor(o[h][e], st);
  }
  if (lane < LPRV) {
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < EV; ++e) sm_o[(wave * G + h) * D + lane * EV + e] = o[h][e];
  }
  if (lane == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h) { sm_ml[wave * 16 + h] = m_run[h]; sm_ml[wave * 16 + 8 + h] = l_run[h]; }
  }
  __syncthreads();
  float* po = a.part_o + ((size_t)((b * a.Hkv + kvh) * a.S + s) * G) * D;
  for (int i = t; i < G * D; i += ATTN_THREADS) {
    const int h = i / D;
    float mb = sm_ml[h];
#pragma unroll
    for (int w = 1; w < NWAVE; ++w) mb = fmaxf(mb, sm_ml[w * 16 + h]);
    float acc = 0.f;
#pragma unroll
    for (int w = 0; w < NWAVE; ++w) acc = fmaf(__builtin_amdgcn_exp2f((sm_ml[w * 16 + h] - mb) * LOG2E), sm_o[w * G * D + i], acc);
    po[i] = acc;
  }
  if (t < G) {
    float mb = sm_ml[t];
#pragma unroll
    for (int w = 1; w < NWAVE; ++w) mb = fmaxf(mb, sm_ml[w * 16 + t]);
    float ll = 0.f;
#pragma unroll
    for (int w = 0; w < NWAVE; ++w) ll = fmaf(__builtin_amdgcn_exp2f((sm_ml[w * 16 + t] - mb) * LOG2E), sm_ml[w * 16 + 8 + t], ll);
    float* pm = a.part_ml + ((size_t)((b * a.Hkv + kvh) * a.S + s) * 2) * G;
    pm[t] = mb;
    pm[G + t] = ll;
  }
}

template <int D, int G, bool BF16>
__global__ __launch_bounds__(ATTN_THREADS) TKV_WPE void k_attn_tiered(const AttnArgs a) {
  constexpr int GP = GPad<G>::v;
  __shared__ __attribute__((aligned(16))) float pbuf[NWAVE * 64 * GP];
  __shared__ float sm_o[NWAVE * G * D];
  __shared__ float sm_ml[NWAVE * 16];
  const int s = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  int nF, nQ;
  if (a.B <= ATTN_ARG_SEQS) { nF = a.nF[b]; nQ = a.nQ[b]; }
  else { nF = a.cnt[b * CNT_N + C_NF]; nQ = a.cnt[b * CNT_N + C_NQ]; }
  const int cf = (nF + TB - 1) / TB, cq = (nQ + TB - 1) / TB, ns = cf + cq;
  if (s >= ns) return;
  if (s < cf) {
    const int j0 = s * TB;
    attn_block<D, G, BF16 ? F_BF16 : F_F32, BF16>(a, sm_o, sm_ml, pbuf, b, kvh, s, min(TB, nF - j0), a.f_loc + (size_t)b * a.Nmax + j0);
  } else {
    const int j0 = (s - cf) * TB;
    if (a.t2fmt == 0) attn_block<D, G, Q_INT8, BF16>(a, sm_o, sm_ml, pbuf, b, kvh, s, min(TB, nQ - j0), a.q_loc + (size_t)b * a.Nmax + j0);
    else attn_block<D, G, Q_INT4, BF16>(a, sm_o, sm_ml, pbuf, b, kvh, s, min(TB, nQ - j0), a.q_loc + (size_t)b * a.Nmax + j0);
  }
}

// ---- finish: global softmax statistics, scores, output ------------------------------------------------------
constexpr int FIN_LDS_FLOATS = 8192;   // room for the (m, l) of all splits of one sequence: Hkv * S * 2 * G floats

template <int D, int G>
__global__ __launch_bounds__(256) void k_attn_finish(const AttnArgs a, int n_tiles) {
  __shared__ float sm_pm[FIN_LDS_FLOATS];
  __shared__ float M[128], IL[128];
  const int t = threadIdx.x, b = blockIdx.y;
  int nF, nQ;
  if (a.B <= ATTN_ARG_SEQS) { nF = a.nF[b]; nQ = a.nQ[b]; }
  else { nF = a.cnt[b * CNT_N + C_NF]; nQ = a.cnt[b * CNT_N + C_NQ]; }
  const int cf = (nF + TB - 1) / TB, cq = (nQ + TB - 1) / TB, ns = cf + cq;
  const bool is_tile = (int)blockIdx.x < n_tiles;
  if (is_tile && (int)blockIdx.x * 64 >= cf * TB + nQ) return;
  // (m, l) of every split of this sequence: part_ml[b][kvh][s][2][G], s < ns
  const float* pmb = a.part_ml + (size_t)b * a.Hkv * a.S * 2 * G;
  const int per_kvh = ns * 2 * G;
  const bool in_lds = a.Hkv * per_kvh <= FIN_LDS_FLOATS;
  if (in_lds) {
    for (int i = t; i < a.Hkv * per_kvh; i += 256) {
      const int kvh = i / per_kvh, rem = i % per_kvh;
      sm_pm[i] = pmb[(size_t)kvh * a.S * 2 * G + rem];
    }
    __syncthreads();
  }
  if (t < a.Hq) {
    const int kvh = t / G, g = t % G;
    const float* src = in_lds ? (sm_pm + kvh * per_kvh) : (pmb + (size_t)kvh * a.S * 2 * G);
    float mm = -INFINITY;
    for (int k = 0; k < ns; ++k) mm = fmaxf(mm, src[k * 2 * G + g]);
    float ll = 0.f;
    for (int k = 0; k < ns; ++k) ll = fmaf(src[k * 2 * G + G + g], __builtin_amdgcn_exp2f((src[k * 2 * G + g] - mm) * LOG2E), ll);
    M[t] = mm;
    IL[t] = 1.0f / ll;
  }
  __syncthreads();
  if (is_tile) {
    // 64 list entries per workgroup; thread (e, hg) sums the softmax weights of kv heads hg, hg+4, ... (all G members
    // of each), then the four partial sums of an entry are added in the fixed order hg = 0, 1, 2, 3
    const int e = t & 63, hg = t >> 6;
    const int j = blockIdx.x * 64 + e;
    int pos = -1;
    if (j < nF) pos = a.f_pos[(size_t)b * a.Nmax + j];
    else if (j >= cf * TB && j - cf * TB < nQ) pos = a.q_pos[(size_t)b * a.Nmax + (j - cf * TB)];
    float acc = 0.f;
    if (pos >= 0) {
      for (int kvh = hg; kvh < a.Hkv; kvh += 4) {
        float x[G];
#pragma unroll
        for (int g = 0; g < G; ++g) x[g] = a.xs[((size_t)b * a.Hq + kvh * G + g) * a.xs_stride + j];
#pragma unroll
        for (int g = 0; g < G; ++g) acc += __builtin_amdgcn_exp2f((x[g] - M[kvh * G + g]) * LOG2E) * IL[kvh * G + g];
      }
    }
    __syncthreads();          // sm_pm is free now: reuse it for the partial sums
    sm_pm[hg * 64 + e] = acc;
    __syncthreads();
    if (hg == 0 && pos >= 0) {
      const float tot = ((sm_pm[e] + sm_pm[64 + e]) + sm_pm[128 + e]) + sm_pm[192 + e];
      a.score[(size_t)b * a.Nmax + pos] += a.score_scale * tot;
    }
  } else {
    // one workgroup per query head: thread (d, sg) sums the splits sg, sg+NSG, ... of output element d, then the NSG
    // partial sums are added in the fixed order sg = 0, 1, ...
    constexpr int NSG = 256 / D;
    const int hq = blockIdx.x - n_tiles, kvh = hq / G, h = hq % G;
    const int d = t % D, sg = t / D;
    const float* pm = in_lds ? (sm_pm + kvh * per_kvh) : (pmb + (size_t)kvh * a.S * 2 * G);
    const float* pob = a.part_o + ((size_t)(b * a.Hkv + kvh) * a.S * G) * D + h * D + d;
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
      const size_t oi = ((size_t)b * a.Hq + hq) * D + d;
      if (a.out_bf16) ((uint16_t*)a.out)[oi] = f32_to_bf16(tot);
      else ((float*)a.out)[oi] = tot;
    }
  }
}

// ---- dispatch ----------------------------------------------------------------------------------------------
// With a pair of events the launch is timed by the dispatch's own begin / end timestamps (no bracket overhead).
template <int D, int G, bool BF16>
static hipError_t run_tiered(const AttnArgs& a, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  dim3 grid(a.S, a.Hkv, a.B);
  if (ev0 && ev1) hipExtLaunchKernelGGL((k_attn_tiered<D, G, BF16>), grid, dim3(ATTN_THREADS), 0, st, ev0, ev1, 0, a);
  else hipLaunchKernelGGL((k_attn_tiered<D, G, BF16>), grid, dim3(ATTN_THREADS), 0, st, a);
  return hipGetLastError();
}
template <int D, int G, bool BF16>
static hipError_t run_finish(const AttnArgs& a, hipStream_t st) {
  const int tiles = (a.S * TB + 63) / 64;
  hipLaunchKernelGGL((k_attn_finish<D, G>), dim3(tiles + a.Hq, a.B), dim3(256), 0, st, a, tiles);
  return hipGetLastError();
}

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

hipError_t launch_attn_tiered(const AttnArgs& a, int D, int G, bool bf16, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  if (D == 128 && bf16) { TKV_DISPATCH_G(run_tiered, 128, true, a, st, ev0, ev1) }
  if (D == 128 && !bf16) { TKV_DISPATCH_G(run_tiered, 128, false, a, st, ev0, ev1) }
  if (D == 64 && bf16) { TKV_DISPATCH_G(run_tiered, 64, true, a, st, ev0, ev1) }
  if (D == 64 && !bf16) { TKV_DISPATCH_G(run_tiered, 64, false, a, st, ev0, ev1) }
  return hipErrorInvalidValue;
}
hipError_t launch_attn_finish(const AttnArgs& a, int D, int G, hipStream_t st) {
  if (D == 128) { TKV_DISPATCH_G(run_finish, 128, true, a, st) }
  if (D == 64) { TKV_DISPATCH_G(run_finish, 64, true, a, st) }
  return hipErrorInvalidValue;
}

}  // namespace tkv
