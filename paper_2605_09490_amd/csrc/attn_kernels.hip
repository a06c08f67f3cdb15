// Decode attention over the tiered KV cache, with cumulative-score emission (Eq. 1, Eq. 2-3 of the paper).
//
// Two kernels per layer call:
//   attn_split  : grid (S, Hkv, B).  Block (s, kvh, b) owns TOK_PER_BLOCK consecutive entries of one of the two
//                 per-sequence lists -- F (T0 u T1 rows at full precision, ascending position) or Q (T2 rows,
//                 int8 / int4 codes dequantised in registers).  T3 positions are in neither list.  The block
//                 streams the K rows (phase 1: logits for the G query heads of the kv head, kept in LDS),
//                 takes an exact block-local softmax (phase 2), then streams the V rows (phase 3).  It leaves a
//                 split partial (m, l, o[G][D]) and the scaled logits of its entries.
//   attn_finish : merges the split partials into out[B, Hq, D] and turns the stored logits into softmax weights
//                 with the global (m, l) of every head, summed over all query heads in a fixed order into
//                 score[b, pos].
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
constexpr int TPW = TB / NWAVE;  // list entries per wave

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
  return __builtin_amdgcn_update_dpp(0.f, x, CTRL, 0xf, 0xf, false);
}

// sum over aligned groups of LPR consecutive lanes; every lane of the group receives the total
template <int LPR>
__device__ __forceinline__ float group_sum(float x) {
  if constexpr (LPR >= 2) x += dpp_f<0xB1>(x);    // quad_perm [1,0,3,2]
  if constexpr (LPR >= 4) x += dpp_f<0x4E>(x);    // quad_perm [2,3,0,1]
  if constexpr (LPR >= 8) x += dpp_f<0x141>(x);   // row_half_mirror
  if constexpr (LPR >= 16) x += dpp_f<0x140>(x);  // row_mirror
  if constexpr (LPR >= 32) x += __shfl_xor(x, 16);
  return x;
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
  return x;
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

// ---- phase 2, common to F and Q blocks -------------------------------------------------------------------
// lg[t][h] holds q_h . k_t (Q blocks: times the row's K scale).  On return lg[t][h] holds
// p = exp(x - m_block) (0 for t >= ntok), the scaled logits are in xs, and (m, l) in part_ml.
template <int G>
__device__ __forceinline__ void softmax_phase(const AttnArgs& a, float* lg, float* red, int b, int kvh, int s, int ntok) {
  constexpr int GP = GPad<G>::v;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const bool valid = t < ntok;
  float x[G], m[G], p[G];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    x[h] = valid ? lg[t * GP + h] * a.softmax_scale : -INFINITY;
    m[h] = wave_max(x[h]);
  }
  if (lane == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h) red[wave * 8 + h] = m[h];
  }
  __syncthreads();
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float mm = red[h];
#pragma unroll
    for (int w = 1; w < NWAVE; ++w) mm = fmaxf(mm, red[w * 8 + h]);
    m[h] = mm;
    p[h] = valid ? __builtin_amdgcn_exp2f((x[h] - mm) * LOG2E) : 0.f;
  }
  float l[G];
#pragma unroll
  for (int h = 0; h < G; ++h) l[h] = wave_sum(p[h]);
  if (lane == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h) red[32 + wave * 8 + h] = l[h];
  }
#pragma unroll
  for (int h = 0; h < G; ++h) lg[t * GP + h] = p[h];
  if (valid) {
    const size_t base = ((size_t)(b * a.Hkv + kvh) * G) * a.xs_stride + (size_t)s * TB + t;
#pragma unroll
    for (int h = 0; h < G; ++h) a.xs[base + (size_t)h * a.xs_stride] = x[h];
  }
  __syncthreads();
  if (t < G) {
    float ll = 0.f;
#pragma unroll
    for (int w = 0; w < NWAVE; ++w) ll += red[32 + w * 8 + t];
    float* pm = a.part_ml + ((size_t)((b * a.Hkv + kvh) * a.S + s) * 2) * G;
    float mm = red[t];
#pragma unroll
    for (int w = 1; w < NWAVE; ++w) mm = fmaxf(mm, red[w * 8 + t]);
    pm[t] = mm;
    pm[G + t] = ll;
  }
}

// sum the per-lane output slices over the RPW row groups of a wave, then over the waves, and store the split partial
template <int D, int G, int LPR, int EPL>
__device__ __forceinline__ void reduce_store_o(const AttnArgs& a, float (&o)[G][EPL], float* ored, int b, int kvh, int s) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
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
      for (int e = 0; e < EPL; ++e) ored[(wave * G + h) * D + lane * EPL + e] = o[h][e];
  }
  __syncthreads();
  float* po = a.part_o + ((size_t)((b * a.Hkv + kvh) * a.S + s) * G) * D;
  for (int i = t; i < G * D; i += ATTN_THREADS) {
    float acc = ored[i];
#pragma unroll
    for (int w = 1; w < NWAVE; ++w) acc += ored[w * G * D + i];
    po[i] = acc;
  }
}

// ---- F block: full-precision rows ------------------------------------------------------------------------
template <int D, int G, bool BF16>
__device__ __forceinline__ void attn_f_block(const AttnArgs& a, float* lg, float* ored, float* red,
                                             int b, int kvh, int s, int j0, int ntok) {
  constexpr int ES = BF16 ? 2 : 4;
  constexpr int EPL = 16 / ES;      // elements per lane (one 128-bit load)
  constexpr int LPR = D / EPL;      // lanes per row
  constexpr int RPW = 64 / LPR;     // rows per wave and load instruction
  constexpr int NIT = TPW / RPW;
  constexpr int U = (NIT >= 4) ? 4 : NIT;
  constexpr int GP = GPad<G>::v;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int grp = lane / LPR, r = lane % LPR;
  const uint32_t row_bytes = D * ES;
  const size_t pool_off = (size_t)(b * a.Hkv + kvh) * a.capF * row_bytes;
  const __amdgpu_buffer_rsrc_t rk = make_rsrc(a.fpK + pool_off, (uint32_t)a.capF * row_bytes);
  const __amdgpu_buffer_rsrc_t rv = make_rsrc(a.fpV + pool_off, (uint32_t)a.capF * row_bytes);

  // this lane's slice of the G query vectors
  uint32_t qp[G][4];
  {
    const char* qb = (const char*)a.q + ((size_t)(b * a.Hq + kvh * G) * D + r * EPL) * ES;
#pragma unroll
    for (int h = 0; h < G; ++h) {
      u32x4 v = *(const u32x4*)(qb + (size_t)h * D * ES);
      qp[h][0] = v.x; qp[h][1] = v.y; qp[h][2] = v.z; qp[h][3] = v.w;
    }
  }
  // slots of this wave's 64 list entries, one per lane; -1 (=> out-of-range offset, loads return 0) past the end
  const int jj = j0 + wave * TPW + lane;
  const int myloc = (wave * TPW + lane < ntok) ? a.f_loc[(size_t)b * a.Nmax + jj] : -1;

  // phase 1: logits
  for (int it0 = 0; it0 < NIT; it0 += U) {
    u32x4 kr[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tw = (it0 + u) * RPW + grp;
      const int loc = __shfl(myloc, tw);
      kr[u] = __builtin_amdgcn_raw_buffer_load_b128(rk, (uint32_t)loc * row_bytes + r * 16, 0, 2);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float x[G];
      const uint32_t kw[4] = {kr[u].x, kr[u].y, kr[u].z, kr[u].w};
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float acc = 0.f;
        if constexpr (BF16) {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, kw[c]), __builtin_bit_cast(bf16x2, qp[h][c]), acc, false);
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c) acc = fmaf(__builtin_bit_cast(float, kw[c]), __builtin_bit_cast(float, qp[h][c]), acc);
        }
        x[h] = group_sum<LPR>(acc);
      }
      float v = x[0];
#pragma unroll
      for (int h = 1; h < G; ++h) v = (r == h) ? x[h] : v;
      const int tl = wave * TPW + (it0 + u) * RPW + grp;
      if (r < G) lg[tl * GP + r] = v;
    }
  }
  __syncthreads();
  softmax_phase<G>(a, lg, red, b, kvh, s, ntok);
  __syncthreads();

  // phase 3: o += p * v
  float o[G][EPL];
#pragma unroll
  for (int h = 0; h < G; ++h)
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[h][e] = 0.f;
  for (int it0 = 0; it0 < NIT; it0 += U) {
    u32x4 vr[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tw = (it0 + u) * RPW + grp;
      const int loc = __shfl(myloc, tw);
      vr[u] = __builtin_amdgcn_raw_buffer_load_b128(rv, (uint32_t)loc * row_bytes + r * 16, 0, 2);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tl = wave * TPW + (it0 + u) * RPW + grp;
      float p[GP];
#pragma unroll
      for (int c = 0; c < GP; c += 4) {
        const float4 pv = *(const float4*)(lg + tl * GP + c);
        p[c] = pv.x; p[c + 1] = pv.y; p[c + 2] = pv.z; p[c + 3] = pv.w;
      }
      float vf[EPL];
      const uint32_t vw[4] = {vr[u].x, vr[u].y, vr[u].z, vr[u].w};
      if constexpr (BF16) {
#pragma unroll
        for (int c = 0; c < 4; ++c) { vf[2 * c] = bf_lo(vw[c]); vf[2 * c + 1] = bf_hi(vw[c]); }
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) vf[c] = __builtin_bit_cast(float, vw[c]);
      }
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[h][e] = fmaf(p[h], vf[e], o[h][e]);
    }
  }
  reduce_store_o<D, G, LPR, EPL>(a, o, ored, b, kvh, s);
}

// ---- Q block: T2 rows, codes dequantised in registers ----------------------------------------------------------
// INT8: a row is D code bytes + one binary32 scale; 8 codes per lane.  INT4: D/2 bytes + D/32 binary16 scales;
// 8 codes (4 bytes) per lane, so four lanes share a scale group.  Codes are read as unsigned with an offset
// (128 / 8) that is removed once per row: sum q*(u - off) = sum q*u - off * sum q.
template <int D, int G, bool BF16, bool INT4>
__device__ __forceinline__ void attn_q_block(const AttnArgs& a, float* lg, float* ored, float* red,
                                             int b, int kvh, int s, int j0, int ntok) {
  constexpr int ES = BF16 ? 2 : 4;
  constexpr int EPL = 8;
  constexpr int LPR = D / EPL;
  constexpr int RPW = 64 / LPR;
  constexpr int NIT = TPW / RPW;
  constexpr int U = (NIT >= 4) ? 4 : NIT;
  constexpr int GP = GPad<G>::v;
  constexpr float OFF = INT4 ? 8.f : 128.f;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int grp = lane / LPR, r = lane % LPR;
  const uint32_t cb = a.cb, sb = a.sb;
  const size_t rows_off = (size_t)(b * a.Hkv + kvh) * a.cap2;
  const __amdgpu_buffer_rsrc_t rkc = make_rsrc(a.c2K + rows_off * cb, (uint32_t)a.cap2 * cb);
  const __amdgpu_buffer_rsrc_t rvc = make_rsrc(a.c2V + rows_off * cb, (uint32_t)a.cap2 * cb);
  const __amdgpu_buffer_rsrc_t rks = make_rsrc(a.s2K + rows_off * sb, (uint32_t)a.cap2 * sb);
  const __amdgpu_buffer_rsrc_t rvs = make_rsrc(a.s2V + rows_off * sb, (uint32_t)a.cap2 * sb);
  const uint32_t lane_code_bytes = INT4 ? 4 : 8;

  const int jj = j0 + wave * TPW + lane;
  const int myloc = (wave * TPW + lane < ntok) ? a.q_loc[(size_t)b * a.Nmax + jj] : -1;

  auto load_scale = [&](const __amdgpu_buffer_rsrc_t& rs, int loc) -> float {
    if constexpr (INT4) {
      // binary16 scale of the 32-element group this lane's 16 codes fall in
      const uint32_t off = (uint32_t)loc * sb + (uint32_t)(r >> 2) * 2;
      const uint16_t hbits = __builtin_amdgcn_raw_buffer_load_b16(rs, off, 0, 0);
      return (float)__builtin_bit_cast(_Float16, hbits);
    } else {
      return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, (uint32_t)loc * sb, 0, 0));
    }
  };
  auto unpack = [&](const u32x2& c, float (&f)[EPL]) {
    if constexpr (INT4) {
      const uint32_t w = c.x ^ 0x88888888u;
#pragma unroll
      for (int n = 0; n < 8; ++n) f[n] = (float)((w >> (4 * n)) & 0xFu);
    } else {
      const uint32_t w[2] = {c.x ^ 0x80808080u, c.y ^ 0x80808080u};
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int n = 0; n < 4; ++n) f[i * 4 + n] = (float)((w[i] >> (8 * n)) & 0xFFu);
    }
  };
  auto load_codes = [&](const __amdgpu_buffer_rsrc_t& rc, int loc) -> u32x2 {
    const uint32_t off = (uint32_t)loc * cb + r * lane_code_bytes;
    if constexpr (INT4) {
      return u32x2{__builtin_amdgcn_raw_buffer_load_b32(rc, off, 0, 2), 0u};
    } else {
      return __builtin_amdgcn_raw_buffer_load_b64(rc, off, 0, 2);
    }
  };

  {
    // query slice as binary32, and its sum for the offset correction
    float qf[G][EPL], qs[G];
    const char* qb = (const char*)a.q + ((size_t)(b * a.Hq + kvh * G) * D + r * EPL) * ES;
#pragma unroll
    for (int h = 0; h < G; ++h) {
      if constexpr (BF16) {
        const u32x4 v0 = *(const u32x4*)(qb + (size_t)h * D * ES);
        const uint32_t w[4] = {v0.x, v0.y, v0.z, v0.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) { qf[h][2 * c] = bf_lo(w[c]); qf[h][2 * c + 1] = bf_hi(w[c]); }
      } else {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const float4 v = *(const float4*)(qb + (size_t)h * D * ES + c * 16);
          qf[h][4 * c] = v.x; qf[h][4 * c + 1] = v.y; qf[h][4 * c + 2] = v.z; qf[h][4 * c + 3] = v.w;
        }
      }
      float sacc = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) sacc += qf[h][e];
      qs[h] = sacc;
    }
    for (int it0 = 0; it0 < NIT; it0 += U) {
      u32x2 kr[U];
      float ksc[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int loc = __shfl(myloc, (it0 + u) * RPW + grp);
        kr[u] = load_codes(rkc, loc);
        ksc[u] = load_scale(rks, loc);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float kf[EPL];
        unpack(kr[u], kf);
        float x[G];
#pragma unroll
        for (int h = 0; h < G; ++h) {
          float acc = -OFF * qs[h];
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc = fmaf(qf[h][e], kf[e], acc);
          if constexpr (INT4) acc *= ksc[u];   // per-group scale before the cross-lane sum
          x[h] = group_sum<LPR>(acc);
          if constexpr (!INT4) x[h] *= ksc[u];
        }
        float v = x[0];
#pragma unroll
        for (int h = 1; h < G; ++h) v = (r == h) ? x[h] : v;
        const int tl = wave * TPW + (it0 + u) * RPW + grp;
        if (r < G) lg[tl * GP + r] = v;
      }
    }
  }
  __syncthreads();
  softmax_phase<G>(a, lg, red, b, kvh, s, ntok);
  __syncthreads();

  float o[G][EPL], osub[G];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    osub[h] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[h][e] = 0.f;
  }
  for (int it0 = 0; it0 < NIT; it0 += U) {
    u32x2 vr[U];
    float vsc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int loc = __shfl(myloc, (it0 + u) * RPW + grp);
      vr[u] = load_codes(rvc, loc);
      vsc[u] = load_scale(rvs, loc);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tl = wave * TPW + (it0 + u) * RPW + grp;
      float p[GP];
#pragma unroll
      for (int c = 0; c < GP; c += 4) {
        const float4 pv = *(const float4*)(lg + tl * GP + c);
        p[c] = pv.x; p[c + 1] = pv.y; p[c + 2] = pv.z; p[c + 3] = pv.w;
      }
      float vf[EPL];
      unpack(vr[u], vf);
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float ps = p[h] * vsc[u];
        osub[h] += ps;
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[h][e] = fmaf(ps, vf[e], o[h][e]);
      }
    }
  }
#pragma unroll
  for (int h = 0; h < G; ++h)
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[h][e] = fmaf(-OFF, osub[h], o[h][e]);
  reduce_store_o<D, G, LPR, EPL>(a, o, ored, b, kvh, s);
}

template <int D, int G, bool BF16>
__global__ __launch_bounds__(ATTN_THREADS) void k_attn_split(const AttnArgs a) {
  constexpr int GP = GPad<G>::v;
  __shared__ __attribute__((aligned(16))) float lg[TB * GP];
  __shared__ float ored[NWAVE * G * D];
  __shared__ float red[64];
  const int s = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int nF = a.cnt[b * CNT_N + C_NF], nQ = a.cnt[b * CNT_N + C_NQ];
  const int cf = (nF + TB - 1) / TB, cq = (nQ + TB - 1) / TB;
  if (s < cf) {
    const int j0 = s * TB;
    attn_f_block<D, G, BF16>(a, lg, ored, red, b, kvh, s, j0, min(TB, nF - j0));
  } else if (s < cf + cq) {
    const int j0 = (s - cf) * TB;
    if (a.t2fmt == 0) attn_q_block<D, G, BF16, false>(a, lg, ored, red, b, kvh, s, j0, min(TB, nQ - j0));
    else attn_q_block<D, G, BF16, true>(a, lg, ored, red, b, kvh, s, j0, min(TB, nQ - j0));
  }
}

// ---- finish: merge the splits, write out, accumulate scores -------------------------------------------------------
template <int D, int G, bool BF16>
__global__ __launch_bounds__(ATTN_THREADS) void k_attn_finish(const AttnArgs a, int n_tiles) {
  __shared__ float M[128], IL[128];
  const int t = threadIdx.x, b = blockIdx.y;
  const int nF = a.cnt[b * CNT_N + C_NF], nQ = a.cnt[b * CNT_N + C_NQ];
  const int cf = (nF + TB - 1) / TB, cq = (nQ + TB - 1) / TB, ns = cf + cq;
  const bool is_tile = (int)blockIdx.x < n_tiles;
  if (is_tile && (int)blockIdx.x >= ns) return;
  if (t < a.Hq) {
    const int kvh = t / G, g = t % G;
    const float* pm = a.part_ml + ((size_t)(b * a.Hkv + kvh) * a.S * 2) * G;
    float mm = -INFINITY;
    for (int s = 0; s < ns; ++s) mm = fmaxf(mm, pm[(size_t)s * 2 * G + g]);
    float ll = 0.f;
    for (int s = 0; s < ns; ++s)
      ll += pm[(size_t)s * 2 * G + G + g] * __builtin_amdgcn_exp2f((pm[(size_t)s * 2 * G + g] - mm) * LOG2E);
    M[t] = mm;
    IL[t] = 1.0f / ll;
  }
  __syncthreads();
  if (is_tile) {
    // one list entry per thread: alpha summed over the query heads in the fixed order kv head, then group member
    const int j = blockIdx.x * TB + t;
    int pos = -1;
    if (j < nF) pos = a.f_pos[(size_t)b * a.Nmax + j];
    else if (j >= cf * TB && j - cf * TB < nQ) pos = a.q_pos[(size_t)b * a.Nmax + (j - cf * TB)];
    if (pos < 0) return;
    float acc = 0.f;
    for (int hq = 0; hq < a.Hq; ++hq) {
      const float x = a.xs[((size_t)b * a.Hq + hq) * a.xs_stride + j];
      acc += __builtin_amdgcn_exp2f((x - M[hq]) * LOG2E) * IL[hq];
    }
    a.score[(size_t)b * a.Nmax + pos] += a.score_scale * acc;
  } else {
    const int kvh = blockIdx.x - n_tiles;
    const float* pm = a.part_ml + ((size_t)(b * a.Hkv + kvh) * a.S * 2) * G;
    const float* po = a.part_o + ((size_t)(b * a.Hkv + kvh) * a.S * G) * D;
    for (int i = t; i < G * D; i += ATTN_THREADS) {
      const int h = i / D, hq = kvh * G + h;
      float acc = 0.f;
      for (int s = 0; s < ns; ++s) {
        const float w = __builtin_amdgcn_exp2f((pm[(size_t)s * 2 * G + h] - M[hq]) * LOG2E);
        acc = fmaf(w, po[(size_t)s * G * D + i], acc);
      }
      acc *= IL[hq];
      const size_t oi = ((size_t)b * a.Hq + hq) * D + (i % D);
      if (a.out_bf16) ((uint16_t*)a.out)[oi] = f32_to_bf16(acc);
      else ((float*)a.out)[oi] = acc;
    }
  }
}

// ---- dispatch ----------------------------------------------------------------------------------------------
template <int D, int G, bool BF16>
static hipError_t run_split(const AttnArgs& a, hipStream_t st) {
  dim3 grid(a.S, a.Hkv, a.B);
  hipLaunchKernelGGL((k_attn_split<D, G, BF16>), grid, dim3(ATTN_THREADS), 0, st, a);
  return hipGetLastError();
}
template <int D, int G, bool BF16>
static hipError_t run_finish(const AttnArgs& a, int n_tiles, hipStream_t st) {
  dim3 grid(n_tiles + a.Hkv, a.B);
  hipLaunchKernelGGL((k_attn_finish<D, G, BF16>), grid, dim3(ATTN_THREADS), 0, st, a, n_tiles);
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
#define TKV_DISPATCH(FN, ...)                                           \
  if (D == 128 && bf16) { TKV_DISPATCH_G(FN, 128, true, __VA_ARGS__) }  \
  if (D == 128 && !bf16) { TKV_DISPATCH_G(FN, 128, false, __VA_ARGS__) } \
  if (D == 64 && bf16) { TKV_DISPATCH_G(FN, 64, true, __VA_ARGS__) }    \
  if (D == 64 && !bf16) { TKV_DISPATCH_G(FN, 64, false, __VA_ARGS__) }  \
  return hipErrorInvalidValue;

hipError_t launch_attn_split(const AttnArgs& a, int D, int G, bool bf16, hipStream_t st) {
  TKV_DISPATCH(run_split, a, st)
}
hipError_t launch_attn_finish(const AttnArgs& a, int D, int G, bool bf16, int n_tiles, hipStream_t st) {
  TKV_DISPATCH(run_finish, a, n_tiles, st)
}

}  // namespace tkv
