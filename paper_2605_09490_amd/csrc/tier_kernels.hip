// Tier management on the device (Sec. 3.3 / Algorithm 1 of the paper): append, rank-based tier assignment by
// radix select, plan counting, plan commit (stream compaction of the tier lists by prefix sums, slot
// allocation from per-pool free stacks), and the row movers (copy, encode, decode, gather, scatter).
// One workgroup of PLAN_THREADS threads owns one sequence in the planning kernels; all work is integer.
#include "tkv_internal.h"

namespace tkv {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;

struct Ppm { uint32_t f[4]; uint32_t rule; };

// ---------------------------------------------------------------------------------------------------------
__global__ void k_init_state(DevView v) {
  const int b = blockIdx.x;
  for (int i = threadIdx.x; i < v.Nmax; i += blockDim.x) {
    const size_t o = (size_t)b * v.Nmax + i;
    v.tier[o] = 0; v.tier_new[o] = 0; v.loc[o] = -1; v.hloc[o] = -1; v.score[o] = 0.f;
  }
  // stacks: the top (highest index) pops first, so slots come out in ascending order
  for (int j = threadIdx.x; j < v.cap0; j += blockDim.x) v.free0[(size_t)b * v.cap0 + j] = v.cap0 - 1 - j;
  for (int j = threadIdx.x; j < v.cap1; j += blockDim.x) v.free1[(size_t)b * v.cap1 + j] = v.cap0 + v.cap1 - 1 - j;
  for (int j = threadIdx.x; j < v.cap2; j += blockDim.x) v.free2[(size_t)b * v.cap2 + j] = v.cap2 - 1 - j;
  if (threadIdx.x < CNT_N) {
    int val = 0;
    if (threadIdx.x == C_FREE0) val = v.cap0;
    if (threadIdx.x == C_FREE1) val = v.cap1;
    if (threadIdx.x == C_FREE2) val = v.cap2;
    v.cnt[b * CNT_N + threadIdx.x] = val;
  }
}
hipError_t launch_init_state(const DevView& v, hipStream_t st) {
  hipLaunchKernelGGL(k_init_state, dim3(v.B), dim3(256), 0, st, v);
  return hipGetLastError();
}

// ---- append ------------------------------------------------------------------------------------------------
// New positions enter T0 (Algorithm 1: the cache grows by the generated token; it is inside the recent window).
__global__ void k_append_assign(DevView v, int pos0, int n_new) {
  const int b = blockIdx.x;
  int* cnt = v.cnt + b * CNT_N;
  const int nfree = cnt[C_FREE0], nF = cnt[C_NF], n0 = cnt[C_N0], len = cnt[C_LEN];
  __syncthreads();
  for (int j = threadIdx.x; j < n_new; j += blockDim.x) {
    const int p = pos0 + j;
    if (nfree - 1 - j < 0 || p >= v.Nmax) continue;   // the host checks capacity before launching
    const int slot = v.free0[(size_t)b * v.cap0 + nfree - 1 - j];
    const size_t o = (size_t)b * v.Nmax;
    v.tier[o + p] = 0; v.loc[o + p] = slot; v.hloc[o + p] = -1;
    v.f_pos[o + nF + j] = p; v.f_loc[o + nF + j] = slot; v.f_loc_old[o + nF + j] = slot;
    v.idx[((size_t)0 * v.B + b) * v.Nmax + n0 + j] = p;
  }
  if (threadIdx.x == 0) {
    cnt[C_FREE0] = nfree - n_new; cnt[C_NF] = nF + n_new; cnt[C_N0] = n0 + n_new; cnt[C_LEN] = len + n_new;
  }
}

// k, v: [B][n_new][Hkv][D]; one thread per 16-byte piece of a row
__global__ void k_append_rows(DevView v, int layer, const char* __restrict__ k, const char* __restrict__ vv, int pos0, int n_new) {
  const int row_bytes = v.D * v.es, cpr = row_bytes / 16;
  const long long total = (long long)v.B * n_new * v.Hkv * cpr;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % cpr);
  long long r = i / cpr;
  const int kvh = (int)(r % v.Hkv); r /= v.Hkv;
  const int j = (int)(r % n_new);
  const int b = (int)(r / n_new);
  const int slot = v.loc[(size_t)b * v.Nmax + pos0 + j];
  if (slot < 0 || slot >= v.capP) return;
  const size_t dst = ((((size_t)layer * v.B + b) * v.Hkv + kvh) * v.capP + slot) * row_bytes + (size_t)c * 16;
  const size_t src = (size_t)i * 16;
  *(u32x4*)(v.fpK + dst) = *(const u32x4*)(k + src);
  *(u32x4*)(v.fpV + dst) = *(const u32x4*)(vv + src);
}

// one new token for every layer at once: k, v [L][B][1][Hkv][D]
__global__ void k_append_step(DevView v, const char* __restrict__ k, const char* __restrict__ vv, int pos) {
  const int row_bytes = v.D * v.es, cpr = row_bytes / 16;
  const long long total = (long long)v.L * v.B * v.Hkv * cpr;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % cpr);
  long long r = i / cpr;
  const int kvh = (int)(r % v.Hkv); r /= v.Hkv;
  const int b = (int)(r % v.B);
  const int layer = (int)(r / v.B);
  const int slot = v.loc[(size_t)b * v.Nmax + pos];
  if (slot < 0 || slot >= v.capP) return;
  const size_t dst = ((((size_t)layer * v.B + b) * v.Hkv + kvh) * v.capP + slot) * row_bytes + (size_t)c * 16;
  *(u32x4*)(v.fpK + dst) = *(const u32x4*)(k + (size_t)i * 16);
  *(u32x4*)(v.fpV + dst) = *(const u32x4*)(vv + (size_t)i * 16);
}
static void launch_vnorm(const DevView& v, const void* rows, long long n_rows, int n_new, int lb0, int pos0, hipStream_t st);
static void launch_redundancy(const DevView& v, const void* rows, long long n_rows, int n_new, int lb0, int pos0, hipStream_t st);

hipError_t launch_append_step(const DevView& v, const void* k, const void* v_, int pos, hipStream_t st) {
  hipLaunchKernelGGL(k_append_assign, dim3(v.B), dim3(256), 0, st, v, pos, 1);
  const long long total = (long long)v.L * v.B * v.Hkv * (v.D * v.es / 16);
  hipLaunchKernelGGL(k_append_step, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, v, (const char*)k, (const char*)v_, pos);
  if (v.vnorm) launch_vnorm(v, v_, (long long)v.L * v.B * v.Hkv, 1, 0, pos, st);
  if (v.red) launch_redundancy(v, k, (long long)v.L * v.B * v.Hkv, 1, 0, pos, st);
  return hipGetLastError();
}

hipError_t launch_append(const DevView& v, int layer, const void* k, const void* v_, int pos0, int n_new, bool assign,
                         hipStream_t st) {
  if (assign) hipLaunchKernelGGL(k_append_assign, dim3(v.B), dim3(256), 0, st, v, pos0, n_new);
  const long long total = (long long)v.B * n_new * v.Hkv * (v.D * v.es / 16);
  const int blocks = (int)((total + 255) / 256);
  hipLaunchKernelGGL(k_append_rows, dim3(blocks), dim3(256), 0, st, v, layer, (const char*)k, (const char*)v_, pos0, n_new);
  if (v.vnorm) launch_vnorm(v, v_, (long long)v.B * n_new * v.Hkv, n_new, layer * v.B, pos0, st);
  if (v.red) launch_redundancy(v, k, (long long)v.B * n_new * v.Hkv, n_new, layer * v.B, pos0, st);
  return hipGetLastError();
}

// ---- classify: radix select of the band boundaries ------------------------------------------------------
// key = already-evicted-first | score in value order | position : 1 + 32 + 24 bits, all distinct.  A binary32
// pattern with the sign bit clear gets it set, one with the sign bit set is complemented: unsigned order of the
// results is the order of the values (the penalised scorers go below zero; for non-negative scores it is the order
// of the patterns themselves).
__device__ __forceinline__ uint64_t rank_key(uint8_t tier_prev, float score, int pos) {
  const uint64_t live = tier_prev == 3 ? 0ull : 1ull;
  const uint32_t u = __builtin_bit_cast(uint32_t, score);
  const uint64_t ord = (u & 0x80000000u) ? (uint32_t)~u : (u | 0x80000000u);
  return (live << 56) | (ord << 24) | (uint64_t)pos;
}
constexpr int RANK_KEY_TOP_SHIFT = 56;   // the radix select walks the key in 8-bit digits from here down (the top one has 1 bit)

__device__ void band_counts(const Ppm& p, long long m, long long evicted, long long out[4]) {
  if (p.rule == 1) {
    // Algorithm 1 as printed: a further floor(r * live) evictions among the candidates still in the cache, the
    // other bands as shares of the survivors
    const long long live = m - evicted, n_new = ((long long)p.f[3] * live) / 1000000, s = live - n_new;
    const long long den = 1000000 - (long long)p.f[3];
    const long long n0 = den > 0 ? ((long long)p.f[0] * s) / den : 0, n2 = den > 0 ? ((long long)p.f[2] * s) / den : 0;
    out[0] = n0; out[1] = s - n0 - n2; out[2] = n2; out[3] = evicted + n_new;
    return;
  }
  long long n3 = ((long long)p.f[3] * m) / 1000000, n2 = ((long long)p.f[2] * m) / 1000000;
  long long n0 = ((long long)p.f[0] * m) / 1000000, n1 = m - n0 - n2 - n3;
  long long extra = evicted - n3;
  if (extra > 0) {
    n3 += extra;
    long long t = extra < n2 ? extra : n2; n2 -= t; extra -= t;
    t = extra < n1 ? extra : n1; n1 -= t; extra -= t;
    t = extra < n0 ? extra : n0; n0 -= t; extra -= t;
  }
  out[0] = n0; out[1] = n1; out[2] = n2; out[3] = n3;
}

__global__ __launch_bounds__(PLAN_THREADS) void k_classify(DevView v, int n, Ppm ppm) {
  __shared__ int hist[256];
  __shared__ int sh_e;
  __shared__ unsigned long long sh_prefix;
  __shared__ int sh_k;
  __shared__ unsigned long long sh_thr[3];
  const int b = blockIdx.x, t = threadIdx.x;
  const uint8_t* tier = v.tier + (size_t)b * v.Nmax;
  uint8_t* tnew = v.tier_new + (size_t)b * v.Nmax;
  const float* score = v.score + (size_t)b * v.Nmax;
  const int lo = v.n_prompt + v.k_sink;
  const int hi = n - v.k_window;
  if (hi <= lo) {
    for (int i = t; i < n; i += PLAN_THREADS) tnew[i] = 0;
    return;
  }
  const int m = hi - lo;
  if (t == 0) sh_e = 0;
  __syncthreads();
  int e = 0;
  for (int i = lo + t; i < hi; i += PLAN_THREADS) e += tier[i] == 3;
  if (e) atomicAdd(&sh_e, e);
  __syncthreads();
  long long bc[4];
  band_counts(ppm, m, sh_e, bc);
  // 0-based ranks at which T2, T1 and T0 start
  const long long ranks[3] = {bc[3], bc[3] + bc[2], bc[3] + bc[2] + bc[1]};
  for (int q = 0; q < 3; ++q) {
    const long long k = ranks[q];
    if (k <= 0) { if (t == 0) sh_thr[q] = 0ull; continue; }
    if (k >= m) { if (t == 0) sh_thr[q] = ~0ull; continue; }
    if (t == 0) { sh_prefix = 0ull; sh_k = (int)k; }
    for (int shift = RANK_KEY_TOP_SHIFT; shift >= 0; shift -= 8) {
      if (t < 256) hist[t] = 0;
      __syncthreads();
      const unsigned long long prefix = sh_prefix;
      for (int i = lo + t; i < hi; i += PLAN_THREADS) {
        const uint64_t key = rank_key(tier[i], score[i], i);
        if (shift == RANK_KEY_TOP_SHIFT || (key >> (shift + 8)) == (prefix >> (shift + 8))) atomicAdd(&hist[(key >> shift) & 255], 1);
      }
      __syncthreads();
      if (t < 64) {
        // the digit whose bin holds rank sh_k: wave 0 scans the 256 bins, 4 per lane
        const int kk = sh_k;
        const int c0 = hist[4 * t], c1 = hist[4 * t + 1], c2 = hist[4 * t + 2], c3 = hist[4 * t + 3];
        const int sum = c0 + c1 + c2 + c3;
        int inc = sum;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const int u = __shfl_up(inc, o);
          if (t >= o) inc += u;
        }
        const int exc = inc - sum;
        if (kk >= exc && kk < inc) {     // exactly one lane (the bins hold at least sh_k + 1 keys in total)
          int r = kk - exc, d = 4 * t;
          if (r >= c0) { r -= c0; ++d; if (r >= c1) { r -= c1; ++d; if (r >= c2) { r -= c2; ++d; } } }
          sh_k = r;
          sh_prefix = prefix | ((unsigned long long)d << shift);
        }
      }
      __syncthreads();
    }
    if (t == 0) sh_thr[q] = sh_prefix;   // the key with exactly k smaller keys
  }
  __syncthreads();
  const uint64_t th3 = sh_thr[0], th2 = sh_thr[1], th1 = sh_thr[2];
  for (int i = t; i < n; i += PLAN_THREADS) {
    uint8_t c = 0;
    if (i >= lo && i < hi) {
      const uint64_t key = rank_key(tier[i], score[i], i);
      c = key < th3 ? 3 : key < th2 ? 2 : key < th1 ? 1 : 0;
    }
    tnew[i] = c;
  }
}
hipError_t launch_classify(const DevView& v, int n, const uint32_t* ppm, hipStream_t st) {
  Ppm p; for (int i = 0; i < 4; ++i) p.f[i] = ppm[i];
  p.rule = ppm[4];
  hipLaunchKernelGGL(k_classify, dim3(v.B), dim3(PLAN_THREADS), 0, st, v, n, p);
  return hipGetLastError();
}

// ---- plan counting (no state change) ---------------------------------------------------------------------
__global__ __launch_bounds__(PLAN_THREADS) void k_plan_count(DevView v, int n) {
  __shared__ int c[16];
  const int b = blockIdx.x, t = threadIdx.x;
  if (t < 16) c[t] = 0;
  __syncthreads();
  const uint8_t* tier = v.tier + (size_t)b * v.Nmax;
  const uint8_t* tnew = v.tier_new + (size_t)b * v.Nmax;
  const int* hloc = v.hloc + (size_t)b * v.Nmax;
  // index: 0..8 = M01 M02 M03 M10 M12 M13 M20 M21 M23, 9 = bad, 10..13 = planned tier counts, 14 = M01 with a valid host copy
  int loc[15];
  for (int k = 0; k < 15; ++k) loc[k] = 0;
  for (int i = t; i < n; i += PLAN_THREADS) {
    const int a = tier[i], d = tnew[i];
    if (d > 3) { loc[9]++; continue; }
    loc[10 + d]++;
    if (a == d) continue;
    if (a == 3) { loc[9]++; continue; }
    const int k = a * 3 + (d > a ? d - 1 : d);   // (a,d) -> 0..8 in the order above
    loc[k]++;
    if (a == 0 && d == 1 && hloc[i] >= 0) loc[14]++;
  }
  for (int k = 0; k < 15; ++k) if (loc[k]) atomicAdd(&c[k], loc[k]);
  __syncthreads();
  int* cnt = v.cnt + b * CNT_N;
  if (t < 9) cnt[C_M01 + t] = c[t];
  if (t == 9) cnt[C_BAD] = c[9];
  if (t >= 10 && t < 14) cnt[C_P0 + (t - 10)] = c[t];
  if (t == 14) { cnt[C_M01R] = c[14]; cnt[C_MCOPY] = c[3] + c[14]; }
}
hipError_t launch_plan_count(const DevView& v, int n, hipStream_t st) {
  hipLaunchKernelGGL(k_plan_count, dim3(v.B), dim3(PLAN_THREADS), 0, st, v, n);
  return hipGetLastError();
}

// ---- plan commit -------------------------------------------------------------------------------------------
// Exclusive scan of four packed 4x16-bit counters over the workgroup (chunk counts never exceed 1024).
struct Pack4 { unsigned long long p[4]; };

template <int THREADS>
__device__ __forceinline__ Pack4 block_excl_scan(const Pack4& in, Pack4& total, unsigned long long (*wsum)[4]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  Pack4 inc = in;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const unsigned long long u = __shfl_up(inc.p[k], o);
      if (lane >= o) inc.p[k] += u;
    }
  }
  if (lane == 63) {
#pragma unroll
    for (int k = 0; k < 4; ++k) wsum[wave][k] = inc.p[k];
  }
  __syncthreads();
  Pack4 ex;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    unsigned long long pre = 0, tot = 0;
    for (int w = 0; w < THREADS / 64; ++w) {
      const unsigned long long s = wsum[w][k];
      if (w < wave) pre += s;
      tot += s;
    }
    ex.p[k] = pre + inc.p[k] - in.p[k];
    total.p[k] = tot;
  }
  __syncthreads();
  return ex;
}

__device__ __forceinline__ int fld(unsigned long long p, int k) { return (int)((p >> (16 * k)) & 0xFFFFull); }

// 512 threads: the 13 running ranks, the packed scan and the move-list bookkeeping need more than the 128 registers a
// thread of a 1024-thread workgroup can have (the wider version spilled 170 of them)
constexpr int COMMIT_THREADS = 512;
__global__ __launch_bounds__(COMMIT_THREADS) void k_plan_commit(DevView v, int n) {
  __shared__ unsigned long long wsum[COMMIT_THREADS / 64][4];
  const int b = blockIdx.x, t = threadIdx.x;
  int* cnt = v.cnt + b * CNT_N;
  const size_t o = (size_t)b * v.Nmax;
  int nfree0 = cnt[C_FREE0];
  const int nfree1 = cnt[C_FREE1], nfree2 = cnt[C_FREE2], npend = cnt[C_PEND];
  int* free0 = v.free0 + (size_t)b * v.cap0;
  int* free1 = v.free1 + (size_t)b * v.cap1;
  int* free2 = v.free2 + (size_t)b * v.cap2;
  __syncthreads();
  // HBM slots whose rows were offloaded at the previous migrate are free now (their staged copies have landed)
  for (int j = t; j < npend; j += COMMIT_THREADS) {
    if (nfree0 + j < v.cap0) free0[nfree0 + j] = v.pend[o + j];
  }
  nfree0 += npend;
  if (nfree0 > v.cap0) nfree0 = v.cap0;
  __syncthreads();

  // running totals: t0 t1 t2 t3 | e0 e1 e2 r0i | r0p r1 r2 mcp | md
  // (r0p doubles as the count of rows that need a transfer: each reads one HBM slot that is released a migrate later)
  int run[13];
  for (int k = 0; k < 13; ++k) run[k] = 0;
  const int hbase = v.host_base[b];
  for (int base = 0; base < n; base += COMMIT_THREADS) {
    const int i = base + t;
    const bool in = i < n;
    const int a = in ? v.tier[o + i] : 0, c = in ? v.tier_new[o + i] : 0;
    const bool ch = in && a != c;
    // a row that returns to T1 while the pinned store still holds its bits needs no transfer
    const bool back = ch && a == 0 && c == 1 && v.hloc[o + i] >= 0;
    const int e0 = ch && ((a == 1 && c == 0) || (a == 2 && (c == 0 || c == 1)));
    const int e1 = ch && c == 1;
    const int e2 = ch && c == 2;
    const int r0i = (ch && a == 0 && (c == 2 || c == 3)) || back;
    const int r0p = ch && c == 1 && !back;       // (a == 0 or a == 2): the HBM slot read by the offload
    const int r1 = ch && a == 1;
    const int r2 = ch && a == 2;
    const int m10 = (ch && a == 1 && c == 0) || back;   // copied inside the F slot space
    const int md = ch && a == 2 && (c == 0 || c == 1);
    Pack4 pk;
    pk.p[0] = (unsigned long long)(in && c == 0) | ((unsigned long long)(in && c == 1) << 16) |
              ((unsigned long long)(in && c == 2) << 32) | ((unsigned long long)(in && c == 3) << 48);
    pk.p[1] = (unsigned long long)e0 | ((unsigned long long)e1 << 16) | ((unsigned long long)e2 << 32) |
              ((unsigned long long)r0i << 48);
    pk.p[2] = (unsigned long long)r0p | ((unsigned long long)r1 << 16) | ((unsigned long long)r2 << 32) |
              ((unsigned long long)m10 << 48);
    pk.p[3] = (unsigned long long)md;
    Pack4 tot;
    const Pack4 ex = block_excl_scan<COMMIT_THREADS>(pk, tot, wsum);
    int rk[13], tt[13];
    for (int k = 0; k < 13; ++k) { rk[k] = run[k] + fld(ex.p[k >> 2], k & 3); tt[k] = fld(tot.p[k >> 2], k & 3); }
    // a chunk total of exactly 1024 does not fit a 16-bit field only if > 65535: fine
    if (in) {
      const int old_loc = v.loc[o + i], old_hloc = v.hloc[o + i];
      int new_loc = old_loc, new_hloc = old_hloc, loc_for_old_list = -2;
      int slot0 = -1;
      if (e0) { const int k = nfree0 - 1 - rk[4]; slot0 = (k >= 0) ? free0[k] : -1; }
      if (ch) {
        if (c == 0) {
          new_loc = slot0;
          if (a != 1) new_hloc = -1;             // up from T1: the host copy stays valid
        } else if (c == 1) {
          const int k1 = nfree1 - 1 - rk[5];
          const int s1 = (k1 >= 0) ? free1[k1] : -1;
          new_loc = s1;
          if (back) {
            // streamed: the row is in the pinned store already and nothing is copied
            v.mv10_src[o + rk[11]] = v.streamed ? -1 : old_loc; v.mv10_dst[o + rk[11]] = s1;
            if (v.streamed) v.h_dst[old_hloc] = s1;
          } else {
            const int src0 = (a == 0) ? old_loc : slot0;
            const int hl = hbase + rk[8];
            new_hloc = hl; loc_for_old_list = src0;
            const int gi = hl - v.event_base;
            v.g_seq[gi] = b; v.g_src[gi] = src0; v.g_dst[gi] = s1;
            if (v.streamed) { v.h_seq[hl] = b; v.h_dst[hl] = s1; }
            v.pend[o + rk[8]] = src0;
          }
        } else if (c == 2) {
          const int k2 = nfree2 - 1 - rk[6];
          const int s2 = (k2 >= 0) ? free2[k2] : -1;
          v.mvq_src[o + rk[6]] = old_loc; v.mvq_dst[o + rk[6]] = s2;
          new_loc = s2; new_hloc = -1;
        } else {
          new_loc = -1; new_hloc = -1;
        }
        if (r0i) v.rel0[o + rk[7]] = old_loc;
        if (r1) { v.rel1[o + rk[9]] = old_loc; if (v.streamed) v.h_clr[o + rk[9]] = old_hloc; }
        if (r2) v.rel2[o + rk[10]] = old_loc;
        if (m10 && !back) { v.mv10_src[o + rk[11]] = old_loc; v.mv10_dst[o + rk[11]] = slot0; }
        if (md) { v.mvd_src[o + rk[12]] = old_loc; v.mvd_dst[o + rk[12]] = slot0; }
        v.loc[o + i] = new_loc; v.hloc[o + i] = new_hloc; v.tier[o + i] = (uint8_t)c;
      }
      v.idx[((size_t)c * v.B + b) * v.Nmax + rk[c]] = i;
      if (c == 1 && v.streamed) {
        v.s_pos[o + rk[1]] = i; v.s_loc[o + rk[1]] = new_loc - v.cap0;
      } else if (c <= 1) {
        const int j = v.streamed ? rk[0] : rk[0] + rk[1];
        v.f_pos[o + j] = i; v.f_loc[o + j] = new_loc;
        v.f_loc_old[o + j] = (loc_for_old_list != -2) ? loc_for_old_list : new_loc;
      } else if (c == 2) {
        v.q_pos[o + rk[2]] = i; v.q_loc[o + rk[2]] = new_loc;
      }
    }
    for (int k = 0; k < 13; ++k) run[k] += tt[k];
  }
  __syncthreads();
  // push the released slots above what is left of each stack
  const int h0 = nfree0 - run[4], h1 = nfree1 - run[5], h2 = nfree2 - run[6];
  for (int j = t; j < run[7]; j += COMMIT_THREADS) if (h0 + j >= 0 && h0 + j < v.cap0) free0[h0 + j] = v.rel0[o + j];
  for (int j = t; j < run[9]; j += COMMIT_THREADS) if (h1 + j >= 0 && h1 + j < v.cap1) free1[h1 + j] = v.rel1[o + j];
  for (int j = t; j < run[10]; j += COMMIT_THREADS) if (h2 + j >= 0 && h2 + j < v.cap2) free2[h2 + j] = v.rel2[o + j];
  if (t == 0) {
    cnt[C_NF] = v.streamed ? run[0] : run[0] + run[1]; cnt[C_NQ] = run[2]; cnt[C_NS] = v.streamed ? run[1] : 0;
    cnt[C_N0] = run[0]; cnt[C_N1] = run[1]; cnt[C_N2] = run[2]; cnt[C_N3] = run[3];
    cnt[C_FREE0] = h0 + run[7]; cnt[C_FREE1] = h1 + run[9]; cnt[C_FREE2] = h2 + run[10];
    cnt[C_PEND] = run[8];
  }
}
hipError_t launch_plan_commit(const DevView& v, int n, hipStream_t st) {
  hipLaunchKernelGGL(k_plan_commit, dim3(v.B), dim3(COMMIT_THREADS), 0, st, v, n);
  return hipGetLastError();
}

// ---- row movers ------------------------------------------------------------------------------------------------
// a row of the unified F slot space: HBM pool, or (streamed T1, staging slots) the frame that holds the layer's T1 rows
// (STREAMED is a template argument so that the resident modes keep one wave-uniform base pointer per access)
template <bool STREAMED>
__device__ __forceinline__ char* fp_ptr(const DevView& v, int which, int layer, int b, int kvh, int slot) {
  const size_t rb = (size_t)(v.D * v.es);
  if constexpr (STREAMED) {
    if (slot >= v.cap0)
      return (which ? v.frV : v.frK) + (((size_t)b * v.Hkv + kvh) * v.cap1 + (slot - v.cap0)) * rb;
  }
  return (which ? v.fpV : v.fpK) + ((((size_t)layer * v.B + b) * v.Hkv + kvh) * v.capP + slot) * rb;
}
__device__ __forceinline__ size_t t2_row(const DevView& v, int layer, int b, int kvh, int slot) {
  return (((size_t)layer * v.B + b) * v.Hkv + kvh) * v.cap2 + slot;
}

// Copies inside the F slot space, bits preserved: T1 -> T0 (staging slot -> HBM slot) and T0 -> T1 of rows whose host
// copy is still valid (HBM slot -> staging slot).  grid (pieces, Hkv*2, L*B)
template <bool STREAMED>
__global__ void k_move_copy(DevView v, int layer0) {
  const int lb = blockIdx.z, layer = layer0 + lb / v.B, b = lb % v.B;
  const int kvh = blockIdx.y >> 1, which = blockIdx.y & 1;
  const int cpr = v.D * v.es / 16;
  const int n = v.cnt[b * CNT_N + C_MCOPY];
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  const int j = i / cpr, c = i % cpr;
  if (j >= n) return;
  const int src = v.mv10_src[(size_t)b * v.Nmax + j], dst = v.mv10_dst[(size_t)b * v.Nmax + j];
  if (src < 0 || src >= v.capF || dst < 0 || dst >= v.capF) return;
  *(u32x4*)(fp_ptr<STREAMED>(v, which, layer, b, kvh, dst) + c * 16) = *(const u32x4*)(fp_ptr<STREAMED>(v, which, layer, b, kvh, src) + c * 16);
}

// 8 consecutive elements of a stored row as binary32
__device__ __forceinline__ void load8(const char* row, int e0, int kt, float (&x)[8]) {
  if (kt == 2) {
    const u32x4 w = *(const u32x4*)(row + (size_t)e0 * 2);
    const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const f16x2 h = __builtin_bit_cast(f16x2, u[c]);
      x[2 * c] = (float)h.x;
      x[2 * c + 1] = (float)h.y;
    }
  } else if (kt == 0) {
    const float4 a = *(const float4*)(row + (size_t)e0 * 4), b = *(const float4*)(row + (size_t)e0 * 4 + 16);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  } else {
    const u32x4 w = *(const u32x4*)(row + (size_t)e0 * 2);
    const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      x[2 * c] = __builtin_bit_cast(float, u[c] << 16);
      x[2 * c + 1] = __builtin_bit_cast(float, u[c] & 0xffff0000u);
    }
  }
}
__device__ __forceinline__ uint32_t bf16_rne_bits(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ void store8(char* row, int e0, int kt, const float (&x)[8]) {
  if (kt == 2) {
    u32x4 w;
    uint32_t u[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      f16x2 h;
      h.x = (_Float16)x[2 * c];          // round to nearest even
      h.y = (_Float16)x[2 * c + 1];
      u[c] = __builtin_bit_cast(uint32_t, h);
    }
    w.x = u[0]; w.y = u[1]; w.z = u[2]; w.w = u[3];
    *(u32x4*)(row + (size_t)e0 * 2) = w;
  } else if (kt == 0) {
    *(float4*)(row + (size_t)e0 * 4) = make_float4(x[0], x[1], x[2], x[3]);
    *(float4*)(row + (size_t)e0 * 4 + 16) = make_float4(x[4], x[5], x[6], x[7]);
  } else {
    u32x4 w;
    w.x = bf16_rne_bits(x[0]) | (bf16_rne_bits(x[1]) << 16); w.y = bf16_rne_bits(x[2]) | (bf16_rne_bits(x[3]) << 16);
    w.z = bf16_rne_bits(x[4]) | (bf16_rne_bits(x[5]) << 16); w.w = bf16_rne_bits(x[6]) | (bf16_rne_bits(x[7]) << 16);
    *(u32x4*)(row + (size_t)e0 * 2) = w;
  }
}

// Value-aware scorer: Euclidean norm of appended value rows.  rows: dense [n_rows][D] in the KV type, row r being
// (layer * B + sequence, new token j, kv head) = (lb0 + r / (n_new * Hkv), (r / Hkv) % n_new, r % Hkv); D / 8 lanes
// per row, each sums the squares of its 8 elements in order, then the lanes' sums are added pairwise (1, 2, 4, 8 apart).
__global__ void k_vnorm(DevView v, const char* __restrict__ rows, long long n_rows, int n_new, int lb0, int pos0) {
  const int lpr = v.D / 8;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long r = i / lpr;
  const int c = (int)(i % lpr);
  float ss = 0.f;
  if (r < n_rows) {
    float x[8];
    load8(rows + (size_t)r * v.D * v.es, c * 8, v.kt, x);
#pragma unroll
    for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
  }
  for (int o = 1; o < lpr; o <<= 1) ss += __shfl_xor(ss, o);
  if (r < n_rows && c == 0) {
    const int kvh = (int)(r % v.Hkv), j = (int)((r / v.Hkv) % n_new);
    const long long lb = lb0 + r / ((long long)n_new * v.Hkv);
    if (pos0 + j < v.Nmax) v.vnorm[((size_t)lb * v.Hkv + kvh) * v.Nmax + pos0 + j] = sqrtf(ss);
  }
}
static void launch_vnorm(const DevView& v, const void* rows, long long n_rows, int n_new, int lb0, int pos0, hipStream_t st) {
  const long long total = n_rows * (v.D / 8);
  hipLaunchKernelGGL(k_vnorm, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, v, (const char*)rows, n_rows, n_new, lb0, pos0);
}

// Redundancy-penalised scorers: the clamped cosine of every appended key row with the key row appended before it
// (the previous new row, or for the first new row the row kept from the last append; 0 for position 0 and for
// all-zero rows).  rows: dense [n_rows][D] as for k_vnorm; D / 8 lanes per row: each accumulates the dot product and the
// two squared norms over its 8 elements in order, then the lanes' sums are added pairwise (1, 2, 4, 8 apart).
__global__ void k_redundancy(DevView v, const char* __restrict__ rows, long long n_rows, int n_new, int lb0, int pos0) {
  const int lpr = v.D / 8;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long r = i / lpr;
  const int c = (int)(i % lpr);
  float dot = 0.f, na = 0.f, nb = 0.f;
  bool has_prev = false;
  if (r < n_rows) {
    const int kvh = (int)(r % v.Hkv), j = (int)((r / v.Hkv) % n_new);
    const long long lb = lb0 + r / ((long long)n_new * v.Hkv);
    float x[8], y[8];
    load8(rows + (size_t)r * v.D * v.es, c * 8, v.kt, x);
    has_prev = j > 0 || pos0 > 0;
    if (j > 0) load8(rows + (size_t)(r - v.Hkv) * v.D * v.es, c * 8, v.kt, y);
    else if (pos0 > 0) load8(v.last_k + ((size_t)lb * v.Hkv + kvh) * v.D * v.es, c * 8, v.kt, y);
    if (has_prev) {
#pragma unroll
      for (int e = 0; e < 8; ++e) { dot = fmaf(x[e], y[e], dot); na = fmaf(x[e], x[e], na); nb = fmaf(y[e], y[e], nb); }
    }
  }
  for (int o = 1; o < lpr; o <<= 1) { dot += __shfl_xor(dot, o); na += __shfl_xor(na, o); nb += __shfl_xor(nb, o); }
  if (r < n_rows && c == 0) {
    const int kvh = (int)(r % v.Hkv), j = (int)((r / v.Hkv) % n_new);
    const long long lb = lb0 + r / ((long long)n_new * v.Hkv);
    const float den = sqrtf(na) * sqrtf(nb);
    const float rho = (has_prev && den > 0.f) ? fmaxf(dot / den, 0.f) : 0.f;
    if (pos0 + j < v.Nmax) v.red[((size_t)lb * v.Hkv + kvh) * v.Nmax + pos0 + j] = rho;
  }
}
// ... and the last new row of every (layer, sequence, kv head) kept for the next append (a launch of its own: the
// kernel above still reads the previous one)
__global__ void k_keep_last_key(DevView v, const char* __restrict__ rows, long long n_groups, int n_new, int lb0) {
  const int cpr = v.D * v.es / 16;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_groups * cpr) return;
  const long long gidx = i / cpr;                     // (lb - lb0, kvh)
  const int c = (int)(i % cpr), kvh = (int)(gidx % v.Hkv);
  const long long lbr = gidx / v.Hkv;
  const long long r = (lbr * n_new + (n_new - 1)) * v.Hkv + kvh;
  *(u32x4*)(v.last_k + (((size_t)(lb0 + lbr)) * v.Hkv + kvh) * v.D * v.es + (size_t)c * 16) =
      *(const u32x4*)(rows + (size_t)r * v.D * v.es + (size_t)c * 16);
}
static void launch_redundancy(const DevView& v, const void* rows, long long n_rows, int n_new, int lb0, int pos0, hipStream_t st) {
  const long long total = n_rows * (v.D / 8);
  hipLaunchKernelGGL(k_redundancy, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, v, (const char*)rows, n_rows, n_new, lb0, pos0);
  const long long groups = n_rows / n_new, t2 = groups * (v.D * v.es / 16);
  hipLaunchKernelGGL(k_keep_last_key, dim3((unsigned)((t2 + 255) / 256)), dim3(256), 0, st, v, (const char*)rows, groups, n_new, lb0);
}

// -> T2: encode the current stored row.  D/8 lanes per row (8 elements each), 64/(D/8) rows per wave.
// grid (pieces, Hkv*2, L*B).  All arithmetic in binary32, round-to-nearest-even, true division.
template <bool STREAMED>
__global__ __launch_bounds__(256) void k_move_quant(DevView v, int layer0) {
  const int lb = blockIdx.z, layer = layer0 + lb / v.B, b = lb % v.B;
  const int kvh = blockIdx.y >> 1, which = blockIdx.y & 1;
  const int lane = threadIdx.x & 63, lpr = v.D / 8, rpw = 64 / lpr;
  const int g = lane / lpr, r = lane % lpr;
  const int j = (blockIdx.x * 4 + (threadIdx.x >> 6)) * rpw + g;
  const int n = v.cnt[b * CNT_N + C_M02] + v.cnt[b * CNT_N + C_M12];
  const bool act = j < n;
  int src = -1, dst = -1;
  if (act) { src = v.mvq_src[(size_t)b * v.Nmax + j]; dst = v.mvq_dst[(size_t)b * v.Nmax + j]; }
  const bool ok = act && src >= 0 && src < v.capF && dst >= 0 && dst < v.cap2;
  float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (ok) load8(fp_ptr<STREAMED>(v, which, layer, b, kvh, src), r * 8, v.kt, x);
  float a = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) a = fmaxf(a, fabsf(x[e]));
  // absmax over the row (int8: all lanes of the row) or over the 32-element group (int4: 4 lanes)
  const int span = v.t2fmt == 0 ? lpr : 4;
  for (int o = 1; o < span; o <<= 1) a = fmaxf(a, __shfl_xor(a, o));
  if (!ok) return;
  const size_t r2 = t2_row(v, layer, b, kvh, dst);
  char* codes = (which ? v.c2V : v.c2K) + r2 * v.cb;
  char* scales = (which ? v.s2V : v.s2K) + r2 * v.sb;
  if (v.t2fmt == 0) {
    const float scale = a / 127.0f;
    uint32_t w[2] = {0u, 0u};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float q = 0.f;
      if (scale > 0.f) q = fminf(fmaxf(rintf(x[e] / scale), -127.f), 127.f);
      w[e >> 2] |= ((uint32_t)((int)q & 0xFF)) << (8 * (e & 3));
    }
    *(uint2*)(codes + r * 8) = make_uint2(w[0], w[1]);
    if (r == 0) *(float*)scales = scale;
  } else {
    const _Float16 sh = (_Float16)(a / 7.0f);
    const float scale = (float)sh;
    uint32_t w = 0u;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float q = 0.f;
      if (scale > 0.f) q = fminf(fmaxf(rintf(x[e] / scale), -7.f), 7.f);
      w |= ((uint32_t)((int)q & 0xF)) << (4 * e);
    }
    *(uint32_t*)(codes + r * 4) = w;
    if ((r & 3) == 0) ((uint16_t*)scales)[r >> 2] = __builtin_bit_cast(uint16_t, sh);
  }
}

// T2 -> T0 (and the HBM stop-over of T2 -> T1): binary32 product code*scale, rounded to the KV dtype.
__global__ __launch_bounds__(256) void k_move_dequant(DevView v) {
  const int lb = blockIdx.z, layer = lb / v.B, b = lb % v.B;
  const int kvh = blockIdx.y >> 1, which = blockIdx.y & 1;
  const int lane = threadIdx.x & 63, lpr = v.D / 8, rpw = 64 / lpr;
  const int g = lane / lpr, r = lane % lpr;
  const int j = (blockIdx.x * 4 + (threadIdx.x >> 6)) * rpw + g;
  const int n = v.cnt[b * CNT_N + C_M20] + v.cnt[b * CNT_N + C_M21];
  if (j >= n) return;
  const int src = v.mvd_src[(size_t)b * v.Nmax + j], dst = v.mvd_dst[(size_t)b * v.Nmax + j];
  if (src < 0 || src >= v.cap2 || dst < 0 || dst >= v.capF) return;
  const size_t r2 = t2_row(v, layer, b, kvh, src);
  const char* codes = (which ? v.c2V : v.c2K) + r2 * v.cb;
  const char* scales = (which ? v.s2V : v.s2K) + r2 * v.sb;
  float x[8];
  if (v.t2fmt == 0) {
    const uint2 w = *(const uint2*)(codes + r * 8);
    const float sc = *(const float*)scales;
    const uint32_t u[2] = {w.x, w.y};
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = (float)(int)(int8_t)((u[e >> 2] >> (8 * (e & 3))) & 0xFF) * sc;
  } else {
    const uint32_t w = *(const uint32_t*)(codes + r * 4);
    const float sc = (float)__builtin_bit_cast(_Float16, ((const uint16_t*)scales)[r >> 2]);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int c = (int)(((w >> (4 * e)) & 0xF) ^ 8) - 8;
      x[e] = (float)c * sc;
    }
  }
  store8(fp_ptr<false>(v, which, layer, b, kvh, dst), r * 8, v.kt, x);     // decoded rows always land in the HBM pool
}

hipError_t launch_moves(const DevView& v, int max10, int maxq, int maxd, hipStream_t st) {
  const int cpr = v.D * v.es / 16;
  const int rpb = 4 * (64 / (v.D / 8));   // rows per workgroup of the encode / decode movers
  if (maxd > 0)
    hipLaunchKernelGGL(k_move_dequant, dim3((maxd + rpb - 1) / rpb, v.Hkv * 2, v.L * v.B), dim3(256), 0, st, v);
  if (max10 > 0)
    hipLaunchKernelGGL(k_move_copy<false>, dim3((max10 * cpr + 255) / 256, v.Hkv * 2, v.L * v.B), dim3(256), 0, st, v, 0);
  if (maxq > 0)
    hipLaunchKernelGGL(k_move_quant<false>, dim3((maxq + rpb - 1) / rpb, v.Hkv * 2, v.L * v.B), dim3(256), 0, st, v, 0);
  return hipGetLastError();
}
hipError_t launch_decode_moves(const DevView& v, int maxd, hipStream_t st) {
  const int rpb = 4 * (64 / (v.D / 8));
  if (maxd > 0)
    hipLaunchKernelGGL(k_move_dequant, dim3((maxd + rpb - 1) / rpb, v.Hkv * 2, v.L * v.B), dim3(256), 0, st, v);
  return hipGetLastError();
}
hipError_t launch_moves_layer(const DevView& v, int layer, int max10, int maxq, hipStream_t st) {
  const int cpr = v.D * v.es / 16;
  const int rpb = 4 * (64 / (v.D / 8));
  if (max10 > 0)
    hipLaunchKernelGGL(k_move_copy<true>, dim3((max10 * cpr + 255) / 256, v.Hkv * 2, v.B), dim3(256), 0, st, v, layer);
  if (maxq > 0)
    hipLaunchKernelGGL(k_move_quant<true>, dim3((maxq + rpb - 1) / rpb, v.Hkv * 2, v.B), dim3(256), 0, st, v, layer);
  return hipGetLastError();
}
// streamed T1: the positions that left T1 in the plan just committed give up their entry in the host-row table
__global__ void k_clear_host_rows(DevView v) {
  const int b = blockIdx.y;
  const int* cnt = v.cnt + b * CNT_N;
  const int n = cnt[C_M10] + cnt[C_M12] + cnt[C_M13];
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  const int h = v.h_clr[(size_t)b * v.Nmax + j];
  if (h >= 0) v.h_dst[h] = -1;
}
hipError_t launch_clear_host_rows(const DevView& v, int max_leaving, hipStream_t st) {
  if (max_leaving > 0)
    hipLaunchKernelGGL(k_clear_host_rows, dim3((max_leaving + 255) / 256, v.B), dim3(256), 0, st, v);
  return hipGetLastError();
}

// T0 -> T1, device side of the offload: pack rows [r0, r0+nrows) of this migrate's host-row order into a
// contiguous bounce piece laid out [row][kv head][K|V][D]; the D2H copy then lands them in the pinned store.
template <bool STREAMED>
__global__ void k_gather(DevView v, int layer, int r0, int nrows, char* __restrict__ bounce) {
  const int row_bytes = v.D * v.es, cpr = row_bytes / 16;
  const long long total = (long long)nrows * v.Hkv * 2 * cpr;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % cpr);
  long long r = i / cpr;
  const int which = (int)(r & 1); r >>= 1;
  const int kvh = (int)(r % v.Hkv);
  const int row = (int)(r / v.Hkv);
  const int b = v.g_seq[r0 + row], src = v.g_src[r0 + row];
  if (b < 0 || b >= v.B || src < 0 || src >= v.capF) return;
  *(u32x4*)(bounce + (size_t)i * 16) = *(const u32x4*)(fp_ptr<STREAMED>(v, which, layer, b, kvh, src) + c * 16);
}
// staging side of the prefetch: unpack a bounce piece (same layout) into the rows' staging slots
__global__ void k_scatter(DevView v, int layer, int r0, int nrows, const char* __restrict__ bounce) {
  const int row_bytes = v.D * v.es, cpr = row_bytes / 16;
  const long long total = (long long)nrows * v.Hkv * 2 * cpr;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % cpr);
  long long r = i / cpr;
  const int which = (int)(r & 1); r >>= 1;
  const int kvh = (int)(r % v.Hkv);
  const int row = (int)(r / v.Hkv);
  const int b = v.g_seq[r0 + row], dst = v.g_dst[r0 + row];
  if (b < 0 || b >= v.B || dst < 0 || dst >= v.capF) return;
  *(u32x4*)(fp_ptr<false>(v, which, layer, b, kvh, dst) + c * 16) = *(const u32x4*)(bounce + (size_t)i * 16);
}
// streamed T1: unpack rows [r0, r0+nrows) of the pinned store's row order (one layer's copy of them, same piece
// layout) into the frame; rows whose position is not in T1 any more are skipped
__global__ void k_scatter_frame(DevView v, int r0, int nrows, const char* __restrict__ bounce) {
  const int row_bytes = v.D * v.es, cpr = row_bytes / 16;
  const long long total = (long long)nrows * v.Hkv * 2 * cpr;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % cpr);
  long long r = i / cpr;
  const int which = (int)(r & 1); r >>= 1;
  const int kvh = (int)(r % v.Hkv);
  const int row = (int)(r / v.Hkv);
  const int b = v.h_seq[r0 + row], dst = v.h_dst[r0 + row];
  if (b < 0 || b >= v.B || dst < v.cap0 || dst >= v.capF) return;
  *(u32x4*)(fp_ptr<true>(v, which, 0, b, kvh, dst) + c * 16) = *(const u32x4*)(bounce + (size_t)i * 16);
}
hipError_t launch_scatter_frame(const DevView& v, int r0, int nrows, const char* bounce, hipStream_t st) {
  const long long total = (long long)nrows * v.Hkv * 2 * (v.D * v.es / 16);
  hipLaunchKernelGGL(k_scatter_frame, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, v, r0, nrows, bounce);
  return hipGetLastError();
}
// Re-homing of the pinned store (it is filled by bump allocation and has run out): the rows T1 holds now get the
// host rows host_base[b], host_base[b] + 1, ... in position order, every other position loses its host row, and
// the gather list names each row's staging slot, so the store can be rewritten from the staged copies.
__global__ __launch_bounds__(PLAN_THREADS) void k_rehome(DevView v, int n) {
  __shared__ unsigned long long wsum[PLAN_THREADS / 64][4];
  const int b = blockIdx.x, t = threadIdx.x;
  const size_t o = (size_t)b * v.Nmax;
  const int hbase = v.host_base[b];
  int run = 0;
  for (int base = 0; base < n; base += PLAN_THREADS) {
    const int i = base + t;
    const bool in = i < n;
    const bool f = in && v.tier[o + i] == 1;
    Pack4 pk;
    pk.p[0] = (unsigned long long)f; pk.p[1] = 0; pk.p[2] = 0; pk.p[3] = 0;
    Pack4 tot;
    const Pack4 ex = block_excl_scan<PLAN_THREADS>(pk, tot, wsum);
    if (in) {
      if (f) {
        const int hl = hbase + run + fld(ex.p[0], 0);
        v.hloc[o + i] = hl;
        v.g_seq[hl] = b; v.g_src[hl] = v.loc[o + i]; v.g_dst[hl] = -1;
      } else {
        v.hloc[o + i] = -1;
      }
    }
    run += fld(tot.p[0], 0);
  }
}
hipError_t launch_rehome(const DevView& v, int n, hipStream_t st) {
  hipLaunchKernelGGL(k_rehome, dim3(v.B), dim3(PLAN_THREADS), 0, st, v, n);
  return hipGetLastError();
}
// Streamed T1, a plan that retires T1 rows: the pinned store is rewritten packed while the plan is applied.  After
// plan_commit, number the positions T1 holds now 0, 1, ... per sequence in position order (base2[b] first) and list
// where each one's bits are: in its staging slot of the layer's frame (it was in T1 before, or it returns to T1 with a
// valid host copy), or, for a row that enters with this plan, in the HBM slot plan_commit noted in its move list.
__global__ __launch_bounds__(PLAN_THREADS) void k_repack_number(DevView v, int n, const int* __restrict__ base2,
                                                                int* __restrict__ g2_seq, int* __restrict__ g2_src,
                                                                int* __restrict__ hloc2) {
  __shared__ unsigned long long wsum[PLAN_THREADS / 64][4];
  const int b = blockIdx.x, t = threadIdx.x;
  const size_t o = (size_t)b * v.Nmax;
  const int hbase = base2[b];
  int run = 0;
  for (int base = 0; base < n; base += PLAN_THREADS) {
    const int i = base + t;
    const bool in = i < n;
    const bool f = in && v.tier[o + i] == 1;
    Pack4 pk;
    pk.p[0] = (unsigned long long)f; pk.p[1] = 0; pk.p[2] = 0; pk.p[3] = 0;
    Pack4 tot;
    const Pack4 ex = block_excl_scan<PLAN_THREADS>(pk, tot, wsum);
    if (in) {
      int hl = -1;
      if (f) {
        hl = hbase + run + fld(ex.p[0], 0);
        const int oldh = v.hloc[o + i];
        g2_seq[hl] = b;
        g2_src[hl] = oldh >= v.event_base ? v.g_src[oldh - v.event_base] : v.loc[o + i];
      }
      hloc2[o + i] = hl;
    }
    run += fld(tot.p[0], 0);
  }
}
__global__ void k_repack_apply(DevView v, int n, const int* __restrict__ hloc2) {
  const int b = blockIdx.y, i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) v.hloc[(size_t)b * v.Nmax + i] = hloc2[(size_t)b * v.Nmax + i];
}
hipError_t launch_repack_number(const DevView& v, int n, const int* base2, int* g2_seq, int* g2_src, int* hloc2, hipStream_t st) {
  hipLaunchKernelGGL(k_repack_number, dim3(v.B), dim3(PLAN_THREADS), 0, st, v, n, base2, g2_seq, g2_src, hloc2);
  return hipGetLastError();
}
hipError_t launch_repack_apply(const DevView& v, int n, const int* hloc2, hipStream_t st) {
  hipLaunchKernelGGL(k_repack_apply, dim3((n + 255) / 256, v.B), dim3(256), 0, st, v, n, hloc2);
  return hipGetLastError();
}

// streamed T1, after a re-homing: the table of host rows, rebuilt from the positions' new host rows
__global__ void k_htable_clear(DevView v, int rows) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < rows) { v.h_seq[i] = -1; v.h_dst[i] = -1; }
}
__global__ void k_htable_fill(DevView v, int n) {
  const int b = blockIdx.y, i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const size_t o = (size_t)b * v.Nmax;
  const int h = v.hloc[o + i];
  if (v.tier[o + i] == 1 && h >= 0) { v.h_seq[h] = b; v.h_dst[h] = v.loc[o + i]; }
}
hipError_t launch_rebuild_htable(const DevView& v, int n, int rows, hipStream_t st) {
  hipLaunchKernelGGL(k_htable_clear, dim3((rows + 255) / 256), dim3(256), 0, st, v, rows);
  hipLaunchKernelGGL(k_htable_fill, dim3((n + 255) / 256, v.B), dim3(256), 0, st, v, n);
  return hipGetLastError();
}

hipError_t launch_gather(const DevView& v, int layer, int r0, int nrows, char* bounce, hipStream_t st) {
  const long long total = (long long)nrows * v.Hkv * 2 * (v.D * v.es / 16);
  if (v.streamed) hipLaunchKernelGGL(k_gather<true>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, v, layer, r0, nrows, bounce);
  else hipLaunchKernelGGL(k_gather<false>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, v, layer, r0, nrows, bounce);
  return hipGetLastError();
}
hipError_t launch_scatter(const DevView& v, int layer, int r0, int nrows, const char* bounce, hipStream_t st) {
  const long long total = (long long)nrows * v.Hkv * 2 * (v.D * v.es / 16);
  hipLaunchKernelGGL(k_scatter, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, v, layer, r0, nrows, bounce);
  return hipGetLastError();
}

}  // namespace tkv
