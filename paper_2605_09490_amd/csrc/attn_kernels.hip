// Decode attention over the tiered KV cache, with cumulative-score emission (Eq. 1, Eq. 2-3 of the paper).
//
//   attn_tiered : grid (S, Hkv, B), 4 waves per workgroup.  Workgroup (s, kvh, b) owns TOK_PER_BLOCK consecutive
//                 entries of one of the two per-sequence lists -- F (T0 u T1 rows at full precision, ascending
//                 position) or Q (T2 rows, int8 / int4 codes dequantised in registers); T3 positions are in
//                 neither list.  Every wave is autonomous: it takes 64-entry tiles, streams their K rows
//                 (16-byte loads, one row per group of lanes), reduces the G logits of each row inside the lane
//                 group so that lane i ends up holding the logits of tile entry i, runs an online softmax with
//                 one entry per lane, then streams the V rows into per-lane output slices.  The four waves are
//                 merged through LDS into one split partial (m, l, o[G][D]); the scaled logits go to a scratch
//                 array.  The last workgroup of a (b, kvh) to finish (device-scope counter) merges that pair's
//                 split partials into out[b, kvh*G .. kvh*G+G) and publishes the global (m, 1/l) of its heads.
//   attn_scores : turns the stored logits into softmax weights with the global (m, 1/l), summed over all query
//                 heads in a fixed order, into score[b, pos].
// The split boundaries and the fp32 summation order depend only on the lists' logical order, never on whether a
// row lives in the HBM pool or the staging buffer (both are one slot space), which is what makes T1 placement
// bit-invisible (Prop. 1).  No MFMA: the path is bound by HBM, and the per-row work is G dot products.
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

enum Mode : int { F_BF16 = 0, F_F32 = 1, Q_INT8 = 2, Q_INT4 = 3 };

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
  return __builtin_amdgcn_update_dpp(0.f, x, CTRL, 0xf, 0xf, false);
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
// Split partials travel between workgroups inside one launch.  They are written and read with relaxed
// device-scope atomics (coherent across the chip's L2 slices by themselves), the writer waits for its stores to
// complete before it takes a ticket, and the reader only starts after it has seen the last ticket; no
// cache-wide release/acquire fence is needed for data that is only ever touched this way.
__device__ __forceinline__ void st_dev(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_dev(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// a value every lane holds identically, moved to a scalar register
__device__ __forceinline__ float uniform(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, x)));
}
// whole-wave reductions: 16-lane rows by DPP, then the four row results through scalar registers
__device__ __forceinline__ float wave_max(float x) {
  x = fmaxf(x, dpp_f<0xB1>(x)); x = fmaxf(x, dpp_f<0x4E>(x)); x = fmaxf(x, dpp_f<0x141>(x)); x = fmaxf(x, dpp_f<0x140>(x));
  return fmaxf(fmaxf(rdlane(x, 0), rdlane(x, 16)), fmaxf(rdlane(x, 32), rdlane(x, 48)));
}
__device__ __forceinline__ float wave_sum(float x) {
  x = group_sum<16>(x);
  return (rdlane(x, 0) + rdlane(x, 16)) + (rdlane(x, 32) + rdlane(x, 48));
}

__device__ __forceinline__ float bf_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __builtin_bit_cast(float, u & 0xffff0000u); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <int G>
struct GPad { static constexpr int v = (G <= 4) ? 4 : 8; };

// one row's worth of registers for one lane
template <Mode M> struct RowRegs;
template <> struct RowRegs<F_BF16> { u32x4 d; };
template <> struct RowRegs<F_F32> { u32x4 d; };
template <> struct RowRegs<Q_INT8> { u32x2 d; float sc; };
template <> struct RowRegs<Q_INT4> { uint32_t d; float sc; };

template <int D, Mode M>
struct Geo {
  static constexpr bool IS_Q = (M == Q_INT8 || M == Q_INT4);
  static constexpr int EPL = (M == F_F32) ? 4 : 8;   // elements of a row per lane
  static constexpr int LPR = D / EPL;                // lanes per row
  static constexpr int NIT = LPR;                    // wave-wide loads per 64-entry tile (64/LPR rows each)
  static constexpr float OFF = (M == Q_INT4) ? 8.f : 128.f;
};

struct RowSrc {
  __amdgpu_buffer_rsrc_t data, scale;
  uint32_t row_bytes, scale_bytes;
};

// loc == -1 gives an offset beyond the buffer: such loads return zeros
template <int D, Mode M>
__device__ __forceinline__ RowRegs<M> load_row(const RowSrc& s, int loc, int r) {
  RowRegs<M> out;
  if constexpr (M == F_BF16 || M == F_F32) {
    out.d = __builtin_amdgcn_raw_buffer_load_b128(s.data, (uint32_t)loc * s.row_bytes + r * 16, 0, 2);
  } else if constexpr (M == Q_INT8) {
    out.d = __builtin_amdgcn_raw_buffer_load_b64(s.data, (uint32_t)loc * s.row_bytes + r * 8, 0, 2);
    out.sc = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(s.scale, (uint32_t)loc * s.scale_bytes, 0, 0));
  } else {
    out.d = __builtin_amdgcn_raw_buffer_load_b32(s.data, (uint32_t)loc * s.row_bytes + r * 4, 0, 2);
    const uint16_t hb = __builtin_amdgcn_raw_buffer_load_b16(s.scale, (uint32_t)loc * s.scale_bytes + (uint32_t)(r >> 2) * 2, 0, 0);
    out.sc = (float)__builtin_bit_cast(_Float16, hb);
  }
  return out;
}

// codes as unsigned values with an offset (128 / 8) that is removed once per row: sum q*(u-off) = sum q*u - off*sum q
template <Mode M>
__device__ __forceinline__ void unpack_codes(const RowRegs<M>& rr, float (&f)[8]) {
  if constexpr (M == Q_INT8) {
    const uint32_t w[2] = {rr.d.x ^ 0x80808080u, rr.d.y ^ 0x80808080u};
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int n = 0; n < 4; ++n) f[i * 4 + n] = (float)((w[i] >> (8 * n)) & 0xFFu);
  } else if constexpr (M == Q_INT4) {
    const uint32_t w = rr.d ^ 0x88888888u;
#pragma unroll
    for (int n = 0; n < 8; ++n) f[n] = (float)((w >> (4 * n)) & 0xFu);
  }
}

// The lane's slice of the G query vectors.  F modes and Q modes with bf16 queries keep the raw 16 bytes (bf16 pairs,
// or 4 floats in F_F32); Q modes with binary32 queries keep 8 floats.  qs is the slice's sum (Q modes).
template <int G, Mode M, bool QBF>
struct QRegs {
  uint32_t qp[G][4];
  float qf[(M == Q_INT8 || M == Q_INT4) && !QBF ? G : 1][8];
  float qs[G];
};

// two code values (exact in bf16: at most 8 significant bits) packed as a bf16 pair
__device__ __forceinline__ uint32_t pack_bf16_pair(float lo, float hi) {
  return (__builtin_bit_cast(uint32_t, hi) & 0xffff0000u) | (__builtin_bit_cast(uint32_t, lo) >> 16);
}

// G logits of one row, reduced over the row's lane group (every lane of the group gets them)
template <int D, int G, Mode M, bool QBF>
__device__ __forceinline__ void row_logits(const RowRegs<M>& rr, const QRegs<G, M, QBF>& q, float (&x)[G]) {
  constexpr int LPR = Geo<D, M>::LPR;
  if constexpr (M == F_BF16 || M == F_F32) {
    const uint32_t kw[4] = {rr.d.x, rr.d.y, rr.d.z, rr.d.w};
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float acc = 0.f;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if constexpr (M == F_BF16)
          acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, kw[c]), __builtin_bit_cast(bf16x2, q.qp[h][c]), acc, false);
        else
          acc = fmaf(__builtin_bit_cast(float, kw[c]), __builtin_bit_cast(float, q.qp[h][c]), acc);
      }
      x[h] = group_sum<LPR>(acc);
    }
  } else {
    float kf[8];
    unpack_codes<M>(rr, kf);
    uint32_t kp[4];
    if constexpr (QBF) {
#pragma unroll
      for (int c = 0; c < 4; ++c) kp[c] = pack_bf16_pair(kf[2 * c], kf[2 * c + 1]);
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float acc = -Geo<D, M>::OFF * q.qs[h];
      if constexpr (QBF) {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, kp[c]), __builtin_bit_cast(bf16x2, q.qp[h][c]), acc, false);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = fmaf(q.qf[h][e], kf[e], acc);
      }
      if constexpr (M == Q_INT4) acc *= rr.sc;      // per-group scale: before the cross-lane sum
      x[h] = group_sum<LPR>(acc);
      if constexpr (M == Q_INT8) x[h] *= rr.sc;     // per-row scale
    }
  }
}

template <int D, int G, Mode M>
__device__ __forceinline__ void row_accumulate(const RowRegs<M>& rr, const float (&p)[GPad<G>::v],
                                               float (&o)[G][Geo<D, M>::EPL], float (&osub)[G]) {
  constexpr int EPL = Geo<D, M>::EPL;
  if constexpr (M == F_BF16) {
    const uint32_t vw[4] = {rr.d.x, rr.d.y, rr.d.z, rr.d.w};
    float vf[8];
#pragma unroll
    for (int c = 0; c < 4; ++c) { vf[2 * c] = bf_lo(vw[c]); vf[2 * c + 1] = bf_hi(vw[c]); }
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[h][e] = fmaf(p[h], vf[e], o[h][e]);
  } else if constexpr (M == F_F32) {
    const uint32_t vw[4] = {rr.d.x, rr.d.y, rr.d.z, rr.d.w};
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[h][e] = fmaf(p[h], __builtin_bit_cast(float, vw[e]), o[h][e]);
  } else {
    float vf[8];
    unpack_codes<M>(rr, vf);
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float ps = p[h] * rr.sc;
      osub[h] += ps;
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[h][e] = fmaf(ps, vf[e], o[h][e]);
    }
  }
}

// ---- one workgroup: TOK_PER_BLOCK entries of list F or Q --------------------------------------------------
// Leaves the workgroup's split partial in part_ml / part_o and the scaled logits in xs.
template <int D, int G, Mode M, bool QBF>
__device__ __forceinline__ void attn_block(const AttnArgs& a, float* sm_o, float* sm_ml, float* pbuf_all,
                                           int b, int kvh, int s, int ntok, const int* loc_list) {
  using GE = Geo<D, M>;
  constexpr int EPL = GE::EPL, LPR = GE::LPR, NIT = GE::NIT;
  constexpr int GP = GPad<G>::v;
  constexpr int U = 4;                     // rows per batch; two batches are kept in flight
  constexpr int NB = NIT / U;              // batches per tile: 2, 4 or 8
  static_assert(NIT % U == 0 && NB % 2 == 0, "tile loads come in an even number of batches of 4");
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int grp = lane / LPR, r = lane % LPR;
  float* pbuf = pbuf_all + wave * 64 * GP;

  RowSrc ks, vs;
  if constexpr (!GE::IS_Q) {
    const uint32_t rb = D * (uint32_t)a.q_es;
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

  // this lane's slice of the G query vectors
  QRegs<G, M, QBF> q;
  {
    constexpr int qes = QBF ? 2 : 4;
    const char* qb = (const char*)a.q + ((size_t)(b * a.Hq + kvh * G) * D + r * EPL) * qes;
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const char* qh = qb + (size_t)h * D * qes;
      if constexpr (M == F_BF16 || M == F_F32) {
        const u32x4 v = *(const u32x4*)qh;
        q.qp[h][0] = v.x; q.qp[h][1] = v.y; q.qp[h][2] = v.z; q.qp[h][3] = v.w;
      } else if constexpr (QBF) {
        const u32x4 v = *(const u32x4*)qh;
        q.qp[h][0] = v.x; q.qp[h][1] = v.y; q.qp[h][2] = v.z; q.qp[h][3] = v.w;
        float sacc = 0.f;
#pragma unroll
        for (int c = 0; c < 4; ++c) sacc += bf_lo(q.qp[h][c]) + bf_hi(q.qp[h][c]);
        q.qs[h] = sacc;
      } else {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const float4 v = *(const float4*)(qh + c * 16);
          q.qf[h][4 * c] = v.x; q.qf[h][4 * c + 1] = v.y; q.qf[h][4 * c + 2] = v.z; q.qf[h][4 * c + 3] = v.w;
        }
        float sacc = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) sacc += q.qf[h][e];
        q.qs[h] = sacc;
      }
    }
  }

  float o[G][EPL], osub[G], m_run[G], l_run[G];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    osub[h] = 0.f; m_run[h] = -INFINITY; l_run[h] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[h][e] = 0.f;
  }

#pragma unroll
  for (int tile = 0; tile < NTILE; ++tile) {
    const int tbase = wave * TPW + tile * 64;          // first entry of the tile, relative to the workgroup
    if (tbase >= ntok) break;                          // wave-uniform
    const bool valid = tbase + lane < ntok;
    // slot of tile entry `lane`; entry grp*LPR + it is loaded by lane group grp at iteration it
    const int myloc = valid ? loc_list[tbase + lane] : -1;

    // Batches 0..NB-1 are the tile's K rows, NB..2NB-1 its V rows; two batches are in flight at any time, so the
    // first V batches are already on their way while the last K batches and the softmax are being computed.
    RowRegs<M> buf0[U], buf1[U];
    auto issue = [&](int k, RowRegs<M> (&dst)[U]) {
      const bool is_k = k < NB;
      const int batch = is_k ? k : k - NB;
      RowSrc src;      // select the descriptor, not the loaded value
      src.data = is_k ? ks.data : vs.data; src.scale = is_k ? ks.scale : vs.scale;
      src.row_bytes = ks.row_bytes; src.scale_bytes = ks.scale_bytes;
#pragma unroll
      for (int u = 0; u < U; ++u) dst[u] = load_row<D, M>(src, __shfl(myloc, grp * LPR + batch * U + u), r);
    };
    float xt[G];
#pragma unroll
    for (int h = 0; h < G; ++h) xt[h] = 0.f;
    auto logits = [&](int k, const RowRegs<M> (&src)[U]) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float x[G];
        row_logits<D, G, M, QBF>(src[u], q, x);
        const int it = k * U + u;
#pragma unroll
        for (int h = 0; h < G; ++h) xt[h] = (r == it) ? x[h] : xt[h];   // lane grp*LPR+it keeps entry grp*LPR+it
      }
    };
    issue(0, buf0);
    issue(1, buf1);
#pragma unroll 1
    for (int k = 0; k < NB; k += 2) {
      logits(k, buf0);
      issue(k + 2, buf0);
      logits(k + 1, buf1);
      issue(k + 3, buf1);
    }
    // ---- online softmax, one entry per lane
    float corr[G];
    {
      const size_t xbase = ((size_t)(b * a.Hq + kvh * G)) * a.xs_stride + (size_t)s * TB + tbase + lane;
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float x = valid ? xt[h] * a.softmax_scale : -INFINITY;
        if (valid) a.xs[xbase + (size_t)h * a.xs_stride] = x;
        const float mn = uniform(fmaxf(m_run[h], wave_max(x)));
        corr[h] = uniform(__builtin_amdgcn_exp2f((m_run[h] - mn) * LOG2E));
        const float p = valid ? __builtin_amdgcn_exp2f((x - mn) * LOG2E) : 0.f;
        l_run[h] = uniform(fmaf(l_run[h], corr[h], wave_sum(p)));
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
        for (int e = 0; e < EPL; ++e) o[h][e] *= corr[h];
      }
    }
    // ---- V rows
    auto accum = [&](int vb, const RowRegs<M> (&src)[U]) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int it = vb * U + u;
        float p[GP];
#pragma unroll
        for (int c = 0; c < GP; c += 4) {
          const float4 pv = *(const float4*)(pbuf + (grp * LPR + it) * GP + c);
          p[c] = pv.x; p[c + 1] = pv.y; p[c + 2] = pv.z; p[c + 3] = pv.w;
        }
        row_accumulate<D, G, M>(src[u], p, o, osub);
      }
    };
#pragma unroll 1
    for (int vb = 0; vb < NB; vb += 2) {
      accum(vb, buf0);
      if (vb + 2 < NB) issue(NB + vb + 2, buf0);
      accum(vb + 1, buf1);
      if (vb + 3 < NB) issue(NB + vb + 3, buf1);
    }
    __builtin_amdgcn_wave_barrier();
  }
  if constexpr (GE::IS_Q) {
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[h][e] = fmaf(-GE::OFF, osub[h], o[h][e]);
  }
  // ---- wave partial: sum the row groups, then merge the four waves through LDS
#pragma unroll
  for (int st = LPR; st < 64; st <<= 1) {
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[h][e] += __shfl_xor(o[h][e], st);
  }
  if (lane < LPR) {
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < EPL; ++e) sm_o[(wave * G + h) * D + lane * EPL + e] = o[h][e];
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
    st_dev(po + i, acc);
  }
  if (t < G) {
    float mb = sm_ml[t];
#pragma unroll
    for (int w = 1; w < NWAVE; ++w) mb = fmaxf(mb, sm_ml[w * 16 + t]);
    float ll = 0.f;
#pragma unroll
    for (int w = 0; w < NWAVE; ++w) ll = fmaf(__builtin_amdgcn_exp2f((sm_ml[w * 16 + t] - mb) * LOG2E), sm_ml[w * 16 + 8 + t], ll);
    float* pm = a.part_ml + ((size_t)((b * a.Hkv + kvh) * a.S + s) * 2) * G;
    st_dev(pm + t, mb);
    st_dev(pm + G + t, ll);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's stores have completed
}

template <int D, int G, bool BF16>
__global__ __launch_bounds__(ATTN_THREADS) void k_attn_tiered(const AttnArgs a) {
  constexpr int GP = GPad<G>::v;
  __shared__ __attribute__((aligned(16))) float pbuf[NWAVE * 64 * GP];
  __shared__ float sm_o[NWAVE * G * D];
  __shared__ float sm_ml[NWAVE * 16];
  __shared__ float sm_fin[16];
  __shared__ int sm_ticket;
  const int s = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z, t = threadIdx.x;
  const int nF = a.cnt[b * CNT_N + C_NF], nQ = a.cnt[b * CNT_N + C_NQ];
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
  // ---- the last workgroup of this (b, kvh) merges the split partials
  __syncthreads();
  if (t == 0) sm_ticket = __hip_atomic_fetch_add(&a.counter[b * a.Hkv + kvh], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  if (sm_ticket != ns - 1) return;
  const float* pm = a.part_ml + ((size_t)(b * a.Hkv + kvh) * a.S * 2) * G;
  const float* pob = a.part_o + ((size_t)(b * a.Hkv + kvh) * a.S * G) * D;
  if (t < G) {
    float mg = -INFINITY;
    for (int k = 0; k < ns; ++k) mg = fmaxf(mg, ld_dev(pm + (size_t)k * 2 * G + t));
    float lg = 0.f;
    for (int k = 0; k < ns; ++k)
      lg = fmaf(ld_dev(pm + (size_t)k * 2 * G + G + t), __builtin_amdgcn_exp2f((ld_dev(pm + (size_t)k * 2 * G + t) - mg) * LOG2E), lg);
    const float il = 1.0f / lg;
    sm_fin[t] = mg; sm_fin[8 + t] = il;
    float* mf = a.ml_final + ((size_t)b * a.Hq + kvh * G + t) * 2;
    mf[0] = mg; mf[1] = il;
  }
  if (t == 0) a.counter[b * a.Hkv + kvh] = 0;
  __syncthreads();
  for (int i = t; i < G * D; i += ATTN_THREADS) {
    const int h = i / D;
    const float mg = sm_fin[h];
    float acc = 0.f;
    for (int k = 0; k < ns; ++k)
      acc = fmaf(__builtin_amdgcn_exp2f((ld_dev(pm + (size_t)k * 2 * G + h) - mg) * LOG2E), ld_dev(pob + (size_t)k * G * D + i), acc);
    acc *= sm_fin[8 + h];
    const size_t oi = ((size_t)b * a.Hq + kvh * G + h) * D + (i % D);
    if (a.out_bf16) ((uint16_t*)a.out)[oi] = f32_to_bf16(acc);
    else ((float*)a.out)[oi] = acc;
  }
}

// ---- scores: one list entry per thread -------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_attn_scores(const AttnArgs a) {
  __shared__ float M[128], IL[128];
  const int t = threadIdx.x, b = blockIdx.y;
  const int nF = a.cnt[b * CNT_N + C_NF], nQ = a.cnt[b * CNT_N + C_NQ];
  const int cf = (nF + TB - 1) / TB;
  const int j = blockIdx.x * 256 + t;
  if ((int)blockIdx.x * 256 >= cf * TB + nQ) return;
  if (t < a.Hq) {
    M[t] = a.ml_final[((size_t)b * a.Hq + t) * 2];
    IL[t] = a.ml_final[((size_t)b * a.Hq + t) * 2 + 1];
  }
  __syncthreads();
  int pos = -1;
  if (j < nF) pos = a.f_pos[(size_t)b * a.Nmax + j];
  else if (j >= cf * TB && j - cf * TB < nQ) pos = a.q_pos[(size_t)b * a.Nmax + (j - cf * TB)];
  if (pos < 0) return;
  // alpha summed over the query heads in the fixed order kv head, then group member
  float acc = 0.f;
  for (int hq = 0; hq < a.Hq; ++hq) {
    const float x = a.xs[((size_t)b * a.Hq + hq) * a.xs_stride + j];
    acc += __builtin_amdgcn_exp2f((x - M[hq]) * LOG2E) * IL[hq];
  }
  a.score[(size_t)b * a.Nmax + pos] += a.score_scale * acc;
}

// ---- dispatch ----------------------------------------------------------------------------------------------
template <int D, int G, bool BF16>
static hipError_t run_tiered(const AttnArgs& a, hipStream_t st) {
  dim3 grid(a.S, a.Hkv, a.B);
  hipLaunchKernelGGL((k_attn_tiered<D, G, BF16>), grid, dim3(ATTN_THREADS), 0, st, a);
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

hipError_t launch_attn_tiered(const AttnArgs& a, int D, int G, bool bf16, hipStream_t st) {
  if (D == 128 && bf16) { TKV_DISPATCH_G(run_tiered, 128, true, a, st) }
  if (D == 128 && !bf16) { TKV_DISPATCH_G(run_tiered, 128, false, a, st) }
  if (D == 64 && bf16) { TKV_DISPATCH_G(run_tiered, 64, true, a, st) }
  if (D == 64 && !bf16) { TKV_DISPATCH_G(run_tiered, 64, false, a, st) }
  return hipErrorInvalidValue;
}
hipError_t launch_attn_scores(const AttnArgs& a, hipStream_t st) {
  const int tiles = (a.S * TB + 255) / 256;
  hipLaunchKernelGGL(k_attn_scores, dim3(tiles, a.B), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace tkv
