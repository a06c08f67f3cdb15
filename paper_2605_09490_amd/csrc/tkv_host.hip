// Host runtime of libtkv: the C ABI of include/tkv.h.  Owns the pools, the per-sequence state, the pinned T1
// store, two side streams (offload: gather + D2H; prefetch: H2D + scatter) and the events that order them
// against attention (Sec. 3.4 of the paper).  All numerical work happens in the kernels; this file only
// validates, sizes, launches and copies.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/tkv.h"
#include "tkv_internal.h"

using namespace tkv;

// ---- scratch of tkv_attend_and_score_noalloc -------------------------------------------------------------------
// The split partials and the scaled logits of one attention call, for callers that may not allocate: a fixed array
// in the library's device image instead of the handle's own allocations.  Every GPU the library runs on holds its own
// copy of the array at its own address (until the process ends); in host code the array's name is only a handle for
// hipGetSymbolAddress, never an address to pass to a kernel.
constexpr size_t NOALLOC_SCRATCH_BYTES = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int RING = 4;
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};   // device address of `scratch` on each device, looked up once per device

// With cfg.device current: the device address of the scratch array on that device (nullptr on failure).
void* scratch_on_device(int device) {
  if (device < 0 || device >= MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[device] = ptr;
  }
  return g_scratch_ptr[device];
}

struct EvPair { hipEvent_t a, b; int64_t bytes; int dir; };  // dir 0 = D2H, 1 = H2D

}  // namespace

// one bounce-buffer piece of a layer's demoted rows: gather -> D2H -> H2D -> scatter
// (nlayers > 1: the same rows of that many consecutive layers, moved by one strided copy each way)
struct XferJob { int layer; int r0; int nrows; int piece; int64_t host_row; bool last_of_layer; int nlayers; };

struct tkv_cache {
  tkv_config cfg{};
  DevView dv{};
  std::string err;
  std::vector<void*> dev_allocs, pin_allocs;
  int G = 0, es = 0;
  int kt = 0;                      // kv_dtype: 0 binary32, 1 bfloat16, 2 binary16
  float score_scale = 0.f, softmax_scale = 0.f;
  // host mirrors
  std::vector<int> len;            // tokens appended per layer
  int n_assigned = 0;              // positions that own a slot
  int n_at_plan = 0;               // n_assigned when the last plan was applied (later positions are T0, the tail of list F)
  std::vector<int> nF, nQ, free0, free1, free2, pend;  // per sequence
  std::vector<int64_t> ntier;      // [4] summed over sequences
  bool plan_pending = false;
  // attention scratch
  float* xs = nullptr; float* part_ml = nullptr; float* part_o = nullptr;
  float* xs_chunk = nullptr; float* ml_chunk = nullptr; float* po_chunk = nullptr;   // the same for chunk launches
  int S_alloc = 0, xs_stride = 0;
  char* static_scratch = nullptr;  // this device's copy of the library's fixed scratch array (tkv_attend_and_score_noalloc)
  // T1 store and transport
  char* hstore = nullptr;
  int64_t host_rows = 0, host_next = 0;
  size_t tok_bytes = 0;            // bytes of one position in one layer: Hkv * 2 * D * es
  hipStream_t sA = nullptr, sB = nullptr;
  hipEvent_t ev_plan = nullptr, ev_piece[RING] = {};
  std::vector<hipEvent_t> ev_ready;
  std::vector<char> layer_wait;
  std::vector<char> layer_enq;      // ev_ready[l] has been recorded for the current re-tiering event
  std::vector<XferJob> jobs;        // transfer pieces of the current event, in layer order
  size_t jobs_next = 0;
  char* bounceA = nullptr; char* bounceB = nullptr;
  size_t bounce_bytes = 0;
  bool transfers_in_flight = false;
  int* pin_cnt = nullptr;          // pinned [B][CNT_N]
  int* pin_base = nullptr;         // pinned [2][B]: first host row per sequence for plan_commit; for a repack
  int* d_host_base = nullptr;
  // streamed T1, repack while a plan is applied: new numbering and gather lists, frame hand-back events
  int* d_base2 = nullptr; int* g2_seq = nullptr; int* g2_src = nullptr; int* hloc2 = nullptr;
  hipEvent_t ev_gath[2] = {nullptr, nullptr};
  // streamed T1: two frames, the layer each holds (-1: none), fill / release events
  bool streamed = false;
  char* frameK[2] = {nullptr, nullptr}; char* frameV[2] = {nullptr, nullptr};
  int frame_layer[2] = {-1, -1};
  bool frame_used[2] = {false, false};   // ev_free[f] has been recorded since the frame was last filled
  hipEvent_t ev_filled[2] = {nullptr, nullptr}, ev_free[2] = {nullptr, nullptr};
  hipStream_t sC = nullptr;        // scatters of the frame fills, so the copies on sB run back to back
  hipEvent_t ev_h2d[RING] = {}, ev_scat[RING] = {};
  bool scat_used[RING] = {};
  std::vector<int> nS;             // per sequence: length of the T1 list
  int64_t fill_piece = 0;
  std::vector<EvPair> copy_events; size_t copy_events_used = 0;
  std::vector<EvPair> prof_events; size_t prof_used = 0;
  std::vector<EvPair> step_events; size_t step_used = 0;   // profile & 2: one pair around every tkv_decode_step
  tkv_stats st{};
};

namespace {

const char* g_static_err = "tkv: NULL handle";

tkv_status fail(tkv_cache* c, tkv_status s, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf;
  return s;
}

#define HIPCHK(c, call)                                                                         \
  do {                                                                                          \
    hipError_t e_ = (call);                                                                     \
    if (e_ != hipSuccess)                                                                       \
      return fail((c), TKV_EDEVICE, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
  } while (0)

void* dev_alloc(tkv_cache* c, size_t bytes) {
  void* p = nullptr;
  if (bytes == 0) bytes = 256;
  if (c->cfg.dev_alloc) p = c->cfg.dev_alloc(bytes, c->cfg.alloc_ctx);
  else if (hipMalloc(&p, bytes) != hipSuccess) p = nullptr;
  if (p) { c->dev_allocs.push_back(p); c->st.device_bytes += (int64_t)bytes; }
  return p;
}
void* pin_alloc(tkv_cache* c, size_t bytes) {
  void* p = nullptr;
  if (bytes == 0) bytes = 256;
  if (c->cfg.pin_alloc) p = c->cfg.pin_alloc(bytes, c->cfg.alloc_ctx);
  else if (hipHostMalloc(&p, bytes, hipHostMallocDefault) != hipSuccess) p = nullptr;
  if (p) { c->pin_allocs.push_back(p); c->st.pinned_bytes += (int64_t)bytes; }
  return p;
}

template <typename T>
bool dalloc(tkv_cache* c, T*& p, size_t count) {
  p = (T*)dev_alloc(c, count * sizeof(T));
  return p != nullptr;
}

bool policy_ok(const tkv_policy* p) {
  return p && (uint64_t)p->f_t0_ppm + p->f_t1_ppm + p->f_t2_ppm + p->f_t3_ppm == 1000000ull && p->count_rule <= 1u;
}

void band_counts_host(const tkv_policy* p, int64_t m, int64_t evicted, int64_t out[4]) {
  if (p->count_rule == TKV_COUNT_ALG1) {
    const int64_t live = m - evicted, n_new = ((int64_t)p->f_t3_ppm * live) / 1000000, s = live - n_new;
    const int64_t den = 1000000 - (int64_t)p->f_t3_ppm;
    const int64_t n0 = den > 0 ? ((int64_t)p->f_t0_ppm * s) / den : 0, n2 = den > 0 ? ((int64_t)p->f_t2_ppm * s) / den : 0;
    out[0] = n0; out[1] = s - n0 - n2; out[2] = n2; out[3] = evicted + n_new;
    return;
  }
  int64_t n3 = ((int64_t)p->f_t3_ppm * m) / 1000000, n2 = ((int64_t)p->f_t2_ppm * m) / 1000000;
  int64_t n0 = ((int64_t)p->f_t0_ppm * m) / 1000000, n1 = m - n0 - n2 - n3;
  int64_t extra = evicted - n3;
  if (extra > 0) {
    n3 += extra;
    int64_t t = std::min(extra, n2); n2 -= t; extra -= t;
    t = std::min(extra, n1); n1 -= t; extra -= t;
    t = std::min(extra, n0); n0 -= t; extra -= t;
  }
  out[0] = n0; out[1] = n1; out[2] = n2; out[3] = n3;
}

int common_length(const tkv_cache* c) {
  int n = c->len[0];
  for (int l = 1; l < c->cfg.n_layers; ++l) if (c->len[l] != n) return -1;
  return n;
}

EvPair* next_pair(std::vector<EvPair>& pool, size_t& used) {
  if (used == pool.size()) {
    EvPair p{};
    if (hipEventCreate(&p.a) != hipSuccess || hipEventCreate(&p.b) != hipSuccess) return nullptr;
    pool.push_back(p);
  }
  return &pool[used++];
}

// waits for the side streams and folds the copy timings into the stats
tkv_status enqueue_job(tkv_cache* c, const XferJob& j) {
  const DevView& v = c->dv;
  const size_t slot_bytes = c->bounce_bytes / RING;
  const size_t bytes = (size_t)j.nrows * c->tok_bytes;
  char* ba = c->bounceA + (size_t)(j.piece % RING) * slot_bytes;
  char* bb = c->bounceB + (size_t)(j.piece % RING) * slot_bytes;
  char* hp = c->hstore + ((size_t)j.layer * c->host_rows + (size_t)j.host_row) * c->tok_bytes;
  if (!next_pair(c->copy_events, c->copy_events_used) || !next_pair(c->copy_events, c->copy_events_used))
    return fail(c, TKV_EDEVICE, "hipEventCreate failed");
  EvPair* ea = &c->copy_events[c->copy_events_used - 2];
  EvPair* eb = &c->copy_events[c->copy_events_used - 1];
  const int nl = j.nlayers;
  const size_t layer_pitch = (size_t)c->host_rows * c->tok_bytes;     // distance of the same host row in the next layer
  ea->dir = 0; eb->dir = 1; ea->bytes = eb->bytes = (int64_t)bytes * nl;
  for (int li = 0; li < nl; ++li) HIPCHK(c, launch_gather(v, j.layer + li, j.r0, j.nrows, ba + (size_t)li * bytes, c->sA));
  HIPCHK(c, hipEventRecord(ea->a, c->sA));
  if (nl == 1) HIPCHK(c, hipMemcpyAsync(hp, ba, bytes, hipMemcpyDeviceToHost, c->sA));
  else HIPCHK(c, hipMemcpy2DAsync(hp, layer_pitch, ba, bytes, bytes, (size_t)nl, hipMemcpyDeviceToHost, c->sA));
  HIPCHK(c, hipEventRecord(ea->b, c->sA));
  if (c->streamed) {
    // the rows stay in the pinned store; the next fill of a layer's frame waits for the layer's last piece
    --c->copy_events_used;
    c->st.d2h_bytes += (int64_t)bytes * nl; c->st.d2h_copies++;
    if (j.last_of_layer)
      for (int li = 0; li < nl; ++li) { HIPCHK(c, hipEventRecord(c->ev_ready[j.layer + li], c->sA)); c->layer_enq[j.layer + li] = 1; }
    return TKV_OK;
  }
  HIPCHK(c, hipEventRecord(c->ev_piece[j.piece % RING], c->sA));
  HIPCHK(c, hipStreamWaitEvent(c->sB, c->ev_piece[j.piece % RING], 0));
  HIPCHK(c, hipEventRecord(eb->a, c->sB));
  if (nl == 1) HIPCHK(c, hipMemcpyAsync(bb, hp, bytes, hipMemcpyHostToDevice, c->sB));
  else HIPCHK(c, hipMemcpy2DAsync(bb, bytes, hp, layer_pitch, bytes, (size_t)nl, hipMemcpyHostToDevice, c->sB));
  HIPCHK(c, hipEventRecord(eb->b, c->sB));
  for (int li = 0; li < nl; ++li) HIPCHK(c, launch_scatter(v, j.layer + li, j.r0, j.nrows, bb + (size_t)li * bytes, c->sB));
  c->st.d2h_bytes += (int64_t)bytes * nl; c->st.h2d_bytes += (int64_t)bytes * nl;
  c->st.d2h_copies++; c->st.h2d_copies++;
  if (j.last_of_layer)
    for (int li = 0; li < nl; ++li) { HIPCHK(c, hipEventRecord(c->ev_ready[j.layer + li], c->sB)); c->layer_enq[j.layer + li] = 1; }
  return TKV_OK;
}

// issues the queued transfer pieces of up to `n_layers` further layers on the side streams
tkv_status pump_transfers(tkv_cache* c, int n_layers) {
  while (c->jobs_next < c->jobs.size() && n_layers > 0) {
    const XferJob& j = c->jobs[c->jobs_next++];
    tkv_status s = enqueue_job(c, j);
    if (s != TKV_OK) return s;
    if (j.last_of_layer) n_layers -= j.nlayers;
  }
  return TKV_OK;
}

tkv_status drain_transfers(tkv_cache* c) {
  if (c->jobs_next < c->jobs.size()) {
    tkv_status s = pump_transfers(c, c->cfg.n_layers);
    if (s != TKV_OK) return s;
  }
  c->jobs.clear(); c->jobs_next = 0;
  if (c->transfers_in_flight) {
    HIPCHK(c, hipStreamSynchronize(c->sA));
    HIPCHK(c, hipStreamSynchronize(c->sB));
    if (c->sC) HIPCHK(c, hipStreamSynchronize(c->sC));
    c->transfers_in_flight = false;
  }
  for (size_t i = 0; i < c->copy_events_used; ++i) {
    float ms = 0.f;
    EvPair& p = c->copy_events[i];
    if (hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) {
      if (p.dir == 0) { c->st.d2h_ms += ms; } else { c->st.h2d_ms += ms; }
    }
  }
  c->copy_events_used = 0;
  std::fill(c->layer_wait.begin(), c->layer_wait.end(), 0);
  std::fill(c->layer_enq.begin(), c->layer_enq.end(), 0);
  return TKV_OK;
}

tkv_status harvest_profile(tkv_cache* c) {
  for (size_t i = 0; i < c->prof_used; ++i) {
    float ms = 0.f;
    HIPCHK(c, hipEventSynchronize(c->prof_events[i].b));
    if (hipEventElapsedTime(&ms, c->prof_events[i].a, c->prof_events[i].b) == hipSuccess) {
      if (c->prof_events[i].dir == 3) {
        // the finishing kernel of a call: its own duration, and the whole call from the first kernel's start
        c->st.attn_finish_ms += ms;
        float call = 0.f;
        if (c->prof_events[i].bytes >= 0 &&
            hipEventElapsedTime(&call, c->prof_events[(size_t)c->prof_events[i].bytes].a, c->prof_events[i].b) == hipSuccess)
          c->st.attn_call_ms += call;
      } else {
        c->st.attn_kernel_ms += ms;
        if (c->prof_events[i].dir != 2) c->st.attn_kernel_launches += 1;   // 2: second launch of the same layer call
      }
    }
  }
  c->prof_used = 0;
  // step pairs: only those whose step has finished (no wait: the call may come in the middle of a timed loop); the
  // pairs still in flight move to the front of the pool
  size_t done = 0;
  while (done < c->step_used && hipEventQuery(c->step_events[done].b) == hipSuccess) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->step_events[done].a, c->step_events[done].b) == hipSuccess) { c->st.step_ms += ms; c->st.steps_timed += 1; }
    ++done;
  }
  if (done > 0) {
    std::rotate(c->step_events.begin(), c->step_events.begin() + done, c->step_events.begin() + c->step_used);
    c->step_used -= done;
  }
  return TKV_OK;
}

// Streamed T1: refill frame f with the T1 rows of `layer` from the pinned store (every row handed out so far; rows
// whose position has left T1 are dropped by the scatter), on the prefetch stream, behind the frame's last reader and
// the layer's last offload.
tkv_status issue_fill(tkv_cache* c, int layer, int f) {
  DevView vv = c->dv;
  vv.frK = c->frameK[f]; vv.frV = c->frameV[f];
  // the copies (prefetch stream) wait for the layer's last offload, the scatters (their own stream) for the frame's
  // last reader: the next layer's rows cross the link while the frame is still being read
  if (c->frame_used[f]) HIPCHK(c, hipStreamWaitEvent(c->sC, c->ev_free[f], 0));
  if (c->layer_wait[layer]) { HIPCHK(c, hipStreamWaitEvent(c->sB, c->ev_ready[layer], 0)); c->layer_wait[layer] = 0; }
  const size_t slot_bytes = c->bounce_bytes / RING;
  const int64_t piece_rows = std::max<int64_t>(1, (int64_t)(slot_bytes / c->tok_bytes));
  EvPair* ev = next_pair(c->copy_events, c->copy_events_used);
  if (!ev) return fail(c, TKV_EDEVICE, "hipEventCreate failed");
  ev->dir = 1; ev->bytes = 0;
  HIPCHK(c, hipEventRecord(ev->a, c->sB));
  for (int64_t r0 = 0; r0 < c->host_next; r0 += piece_rows) {
    const int nrows = (int)std::min<int64_t>(piece_rows, c->host_next - r0);
    const size_t bytes = (size_t)nrows * c->tok_bytes;
    const int slot = (int)(c->fill_piece++ % RING);
    char* bb = c->bounceB + (size_t)slot * slot_bytes;
    if (c->scat_used[slot]) HIPCHK(c, hipStreamWaitEvent(c->sB, c->ev_scat[slot], 0));   // the scatter that read this slot last
    HIPCHK(c, hipMemcpyAsync(bb, c->hstore + ((size_t)layer * c->host_rows + (size_t)r0) * c->tok_bytes, bytes,
                             hipMemcpyHostToDevice, c->sB));
    HIPCHK(c, hipEventRecord(c->ev_h2d[slot], c->sB));
    HIPCHK(c, hipStreamWaitEvent(c->sC, c->ev_h2d[slot], 0));
    HIPCHK(c, launch_scatter_frame(vv, (int)r0, nrows, bb, c->sC));
    HIPCHK(c, hipEventRecord(c->ev_scat[slot], c->sC));
    c->scat_used[slot] = true;
    c->st.h2d_bytes += (int64_t)bytes; c->st.h2d_copies++;
  }
  HIPCHK(c, hipEventRecord(ev->b, c->sB));
  HIPCHK(c, hipEventRecord(c->ev_filled[f], c->sC));
  c->frame_layer[f] = layer;
  c->frame_used[f] = false;
  c->transfers_in_flight = true;
  return TKV_OK;
}

// The pinned store hands out rows in order and has none left: give the rows T1 holds now the rows 0, 1, ... (per
// sequence, in position order) and rewrite the store from their staged copies, one D2H per layer and bounce piece.
// All transfers have been drained, so every T1 row is in its staging slot and nothing reads the store.  T0 rows
// lose their (reusable) host copy.  pin_cnt holds the counters plan_count has just left.
// Streamed T1 has no staged copies: each layer's rows are first brought into a frame (by the old table of host rows),
// packed from there, and the table is rebuilt at the end.
tkv_status rehome_store(tkv_cache* c, int n, hipStream_t st) {
  DevView& v = c->dv;
  const int B = v.B, L = v.L;
  int64_t total = 0;
  for (int b = 0; b < B; ++b) { c->pin_base[b] = (int)total; total += c->pin_cnt[b * CNT_N + C_N1]; }
  HIPCHK(c, hipMemcpyAsync(c->d_host_base, c->pin_base, (size_t)B * sizeof(int), hipMemcpyHostToDevice, st));
  HIPCHK(c, launch_rehome(v, n, st));
  HIPCHK(c, hipEventRecord(c->ev_plan, st));
  HIPCHK(c, hipStreamWaitEvent(c->sA, c->ev_plan, 0));
  if (c->streamed) HIPCHK(c, hipStreamWaitEvent(c->sB, c->ev_plan, 0));
  const size_t slot_bytes = c->bounce_bytes / RING;
  const int64_t piece_rows = std::max<int64_t>(1, (int64_t)(slot_bytes / c->tok_bytes));
  int piece = 0;
  for (int l = 0; l < L; ++l) {
    DevView vl = v;
    if (c->streamed) {
      const int f = l & 1;
      tkv_status fs = issue_fill(c, l, f);
      if (fs != TKV_OK) return fs;
      HIPCHK(c, hipStreamWaitEvent(c->sA, c->ev_filled[f], 0));
      vl.frK = c->frameK[f]; vl.frV = c->frameV[f];
    }
    for (int64_t r0 = 0; r0 < total; r0 += piece_rows, ++piece) {
      const int nrows = (int)std::min<int64_t>(piece_rows, total - r0);
      const size_t bytes = (size_t)nrows * c->tok_bytes;
      char* ba = c->bounceA + (size_t)(piece % RING) * slot_bytes;     // one stream: a ring slot is refilled after its copy
      HIPCHK(c, launch_gather(vl, l, (int)r0, nrows, ba, c->sA));
      HIPCHK(c, hipMemcpyAsync(c->hstore + ((size_t)l * c->host_rows + (size_t)r0) * c->tok_bytes, ba, bytes,
                               hipMemcpyDeviceToHost, c->sA));
      c->st.d2h_bytes += (int64_t)bytes; c->st.d2h_copies++;
    }
    if (c->streamed) { HIPCHK(c, hipEventRecord(c->ev_free[l & 1], c->sA)); c->frame_used[l & 1] = true; }
  }
  HIPCHK(c, hipStreamSynchronize(c->sA));
  if (c->streamed) {
    HIPCHK(c, hipStreamSynchronize(c->sB));
    HIPCHK(c, hipStreamSynchronize(c->sC));
    HIPCHK(c, launch_rebuild_htable(v, n, (int)c->host_rows, st));
    c->frame_layer[0] = c->frame_layer[1] = -1;
  }
  c->host_next = total;
  c->st.n_rehome++;
  return TKV_OK;
}

}  // namespace

extern "C" {

const char* tkv_last_error(const tkv_cache* c) { return c ? c->err.c_str() : g_static_err; }

tkv_status tkv_tier_counts(const tkv_policy* policy, int64_t m, int64_t n_already_evicted, int64_t out[4]) {
  if (!policy_ok(policy) || !out || m < 0 || n_already_evicted < 0 || n_already_evicted > m) return TKV_EINVAL;
  band_counts_host(policy, m, n_already_evicted, out);
  return TKV_OK;
}

tkv_status tkv_create(const tkv_config* cfg, tkv_cache** out) {
  if (out) *out = nullptr;
  if (!cfg || !out) { g_static_err = "tkv_create: NULL argument"; return TKV_EINVAL; }
  auto bad = [&](const char* m) { g_static_err = m; return TKV_EINVAL; };
  if (cfg->n_layers < 1 || cfg->batch < 1 || cfg->n_q_heads < 1 || cfg->n_kv_heads < 1) return bad("tkv_create: sizes must be positive");
  if (cfg->batch * (int64_t)cfg->n_layers > 65535) return bad("tkv_create: n_layers*batch must be <= 65535");
  if (cfg->n_q_heads % cfg->n_kv_heads) return bad("tkv_create: n_q_heads must be a multiple of n_kv_heads");
  const int G = cfg->n_q_heads / cfg->n_kv_heads;
  if (G > MAX_G) return bad("tkv_create: group size n_q_heads/n_kv_heads must be <= 8");
  if (cfg->n_q_heads > 128) return bad("tkv_create: n_q_heads must be <= 128");
  if (cfg->head_dim != 64 && cfg->head_dim != 128) return bad("tkv_create: head_dim must be 64 or 128");
  if (cfg->max_tokens < 1 || cfg->max_tokens >= (1 << 24)) return bad("tkv_create: max_tokens must be in [1, 2^24)");
  if (cfg->kv_dtype < TKV_F32 || cfg->kv_dtype > TKV_F16) return bad("tkv_create: kv_dtype");
  if (cfg->out_dtype < TKV_F32 || cfg->out_dtype > TKV_F16) return bad("tkv_create: out_dtype");
  if (cfg->t2_format != TKV_T2_INT8_ROW && cfg->t2_format != TKV_T2_INT4_G32) return bad("tkv_create: t2_format");
  if (cfg->n_prompt < 0 || cfg->k_sink < 0 || cfg->k_window < 0) return bad("tkv_create: protected sizes must be >= 0");
  if (cfg->t0_rows < 0 || cfg->staging_rows < 0 || cfg->t2_rows < 0 || cfg->host_rows < 0 || cfg->bounce_bytes < 0)
    return bad("tkv_create: capacities must be >= 0");
  if (cfg->prefetch_mode < TKV_PREFETCH_WAIT || cfg->prefetch_mode > TKV_PREFETCH_STREAM) return bad("tkv_create: prefetch_mode");
  if (cfg->scorer < TKV_SCORE_ATTENTION || cfg->scorer > TKV_SCORE_COMBINED) return bad("tkv_create: scorer");
  if (!(cfg->redundancy_weight >= 0.f)) return bad("tkv_create: redundancy_weight must be >= 0");
  if (!(cfg->score_scale >= 0.f) || !(cfg->softmax_scale >= 0.f)) return bad("tkv_create: scales must be >= 0");
  if ((cfg->dev_alloc == nullptr) != (cfg->dev_free == nullptr) || (cfg->pin_alloc == nullptr) != (cfg->pin_free == nullptr))
    return bad("tkv_create: allocator callbacks must come in alloc/free pairs");

  tkv_cache* c = new tkv_cache();
  c->cfg = *cfg;
  c->G = G;
  c->kt = cfg->kv_dtype;
  c->es = c->kt == TKV_F32 ? 4 : 2;
  c->score_scale = cfg->score_scale > 0.f ? cfg->score_scale : 1.0f / ((float)cfg->n_layers * (float)cfg->n_q_heads);
  c->softmax_scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / sqrtf((float)cfg->head_dim);
  auto die = [&](tkv_status s, const char* m) {
    g_static_err = m;
    tkv_destroy(c);
    return s;
  };
  if (hipSetDevice(cfg->device) != hipSuccess) return die(TKV_EDEVICE, "tkv_create: hipSetDevice failed");
  c->static_scratch = (char*)scratch_on_device(cfg->device);
  if (!c->static_scratch) return die(TKV_EDEVICE, "tkv_create: hipGetSymbolAddress of the static scratch array failed");

  DevView& v = c->dv;
  const int L = cfg->n_layers, B = cfg->batch, Hkv = cfg->n_kv_heads, D = cfg->head_dim, N = cfg->max_tokens;
  v.L = L; v.B = B; v.Hq = cfg->n_q_heads; v.Hkv = Hkv; v.G = G; v.D = D; v.Nmax = N;
  v.cap0 = cfg->t0_rows ? cfg->t0_rows : N;
  v.cap1 = cfg->staging_rows ? cfg->staging_rows : N;
  v.cap2 = cfg->t2_rows ? cfg->t2_rows : N;
  v.capF = v.cap0 + v.cap1;
  c->streamed = cfg->prefetch_mode == TKV_PREFETCH_STREAM;
  v.streamed = c->streamed ? 1 : 0;
  v.capP = c->streamed ? v.cap0 : v.capF;
  v.es = c->es;
  v.kt = c->kt;
  v.t2fmt = cfg->t2_format;
  v.cb = cfg->t2_format == TKV_T2_INT8_ROW ? D : D / 2;
  v.sb = cfg->t2_format == TKV_T2_INT8_ROW ? 4 : (D / 32) * 2;
  v.n_prompt = cfg->n_prompt; v.k_sink = cfg->k_sink; v.k_window = cfg->k_window;
  if ((int64_t)v.capF * D * c->es >= (1ll << 31) || (int64_t)v.cap2 * v.cb >= (1ll << 31))
    return die(TKV_EINVAL, "tkv_create: a per-(sequence, kv head) pool must stay below 2 GiB");

  const size_t rows = (size_t)L * B * Hkv;
  const size_t BN = (size_t)B * N;
  bool ok = true;
  ok = ok && dalloc(c, v.fpK, rows * v.capP * D * c->es) && dalloc(c, v.fpV, rows * v.capP * D * c->es);
  ok = ok && dalloc(c, v.c2K, rows * v.cap2 * v.cb) && dalloc(c, v.c2V, rows * v.cap2 * v.cb);
  ok = ok && dalloc(c, v.s2K, rows * v.cap2 * v.sb) && dalloc(c, v.s2V, rows * v.cap2 * v.sb);
  ok = ok && dalloc(c, v.tier, BN) && dalloc(c, v.tier_new, BN) && dalloc(c, v.loc, BN) && dalloc(c, v.hloc, BN);
  ok = ok && dalloc(c, v.score, BN) && dalloc(c, v.f_pos, BN) && dalloc(c, v.f_loc, BN) && dalloc(c, v.f_loc_old, BN);
  ok = ok && dalloc(c, v.q_pos, BN) && dalloc(c, v.q_loc, BN) && dalloc(c, v.idx, 4 * BN) && dalloc(c, v.cnt, (size_t)B * CNT_N);
  ok = ok && dalloc(c, v.free0, (size_t)B * v.cap0) && dalloc(c, v.free1, (size_t)B * v.cap1) && dalloc(c, v.free2, (size_t)B * v.cap2);
  ok = ok && dalloc(c, v.pend, BN) && dalloc(c, v.rel0, BN) && dalloc(c, v.rel1, BN) && dalloc(c, v.rel2, BN);
  ok = ok && dalloc(c, v.mv10_src, BN) && dalloc(c, v.mv10_dst, BN) && dalloc(c, v.mvq_src, BN) && dalloc(c, v.mvq_dst, BN);
  ok = ok && dalloc(c, v.mvd_src, BN) && dalloc(c, v.mvd_dst, BN);
  ok = ok && dalloc(c, v.g_seq, BN) && dalloc(c, v.g_src, BN) && dalloc(c, v.g_dst, BN);
  ok = ok && dalloc(c, c->d_host_base, (size_t)B);
  if (cfg->scorer == TKV_SCORE_VATP || cfg->scorer == TKV_SCORE_COMBINED) ok = ok && dalloc(c, v.vnorm, (size_t)L * B * Hkv * N);
  if (cfg->scorer == TKV_SCORE_REDUNDANCY || cfg->scorer == TKV_SCORE_COMBINED)
    ok = ok && dalloc(c, v.red, (size_t)L * B * Hkv * N) && dalloc(c, v.last_k, (size_t)L * B * Hkv * D * v.es);
  v.host_base = c->d_host_base;
  {
    // one attention workgroup per compute unit: that many per (sequence, kv head) pair, as far as the pairs go round
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, cfg->device) != hipSuccess || cus <= 0) cus = 256;
    c->S_alloc = std::max(1, cus / std::max(1, B * Hkv));
  }
  // every list may end in a partly filled tile; an odd number of 256-byte tiles per row keeps the rows of the heads
  // of one tile from falling on the same memory channels
  c->xs_stride = ((N / TOK_PER_BLOCK + (cfg->prefetch_mode == TKV_PREFETCH_STREAM ? 3 : 2)) | 1) * TOK_PER_BLOCK;
  ok = ok && dalloc(c, c->xs, (size_t)B * v.Hq * c->xs_stride);
  const int launches = c->streamed ? 2 : 1;   // streamed T1: a second attention launch serves the frame
  ok = ok && dalloc(c, c->part_ml, (size_t)B * Hkv * c->S_alloc * launches * 2 * G);
  ok = ok && dalloc(c, c->part_o, (size_t)B * Hkv * c->S_alloc * launches * G * D);
  c->tok_bytes = (size_t)Hkv * 2 * D * c->es;
  c->bounce_bytes = cfg->bounce_bytes ? (size_t)cfg->bounce_bytes : ((size_t)64 << 20);
  if (c->bounce_bytes < RING * c->tok_bytes) c->bounce_bytes = RING * c->tok_bytes;
  ok = ok && dalloc(c, c->bounceA, c->bounce_bytes) && dalloc(c, c->bounceB, c->bounce_bytes);
  c->host_rows = cfg->host_rows ? cfg->host_rows : (int64_t)B * N;
  if (c->streamed) {
    const size_t frame_bytes = (size_t)B * Hkv * v.cap1 * D * c->es;
    for (int f = 0; f < 2; ++f) ok = ok && dalloc(c, c->frameK[f], frame_bytes) && dalloc(c, c->frameV[f], frame_bytes);
    ok = ok && dalloc(c, v.s_pos, BN) && dalloc(c, v.s_loc, BN) && dalloc(c, v.h_clr, BN);
    ok = ok && dalloc(c, v.h_seq, (size_t)c->host_rows) && dalloc(c, v.h_dst, (size_t)c->host_rows);
    ok = ok && dalloc(c, c->d_base2, (size_t)B) && dalloc(c, c->g2_seq, BN) && dalloc(c, c->g2_src, BN) && dalloc(c, c->hloc2, BN);
    if (ok && (hipMemset(v.h_seq, 0xFF, (size_t)c->host_rows * sizeof(int)) != hipSuccess ||
               hipMemset(v.h_dst, 0xFF, (size_t)c->host_rows * sizeof(int)) != hipSuccess))
      return die(TKV_EDEVICE, "tkv_create: state initialisation failed");
    v.frK = c->frameK[0]; v.frV = c->frameV[0];
  }
  if (ok) {
    c->hstore = (char*)pin_alloc(c, (size_t)L * c->host_rows * c->tok_bytes);
    c->pin_cnt = (int*)pin_alloc(c, (size_t)B * CNT_N * sizeof(int));
    c->pin_base = (int*)pin_alloc(c, (size_t)2 * B * sizeof(int));
    ok = c->hstore && c->pin_cnt && c->pin_base;
  }
  if (!ok) return die(TKV_ENOMEM, "tkv_create: an allocation failed");

  c->len.assign(L, 0);
  c->nF.assign(B, 0); c->nQ.assign(B, 0); c->nS.assign(B, 0);
  c->free0.assign(B, v.cap0); c->free1.assign(B, v.cap1); c->free2.assign(B, v.cap2); c->pend.assign(B, 0);
  c->ntier.assign(4, 0);
  c->ev_ready.assign(L, nullptr);
  c->layer_wait.assign(L, 0);
  c->layer_enq.assign(L, 0);
  // default-priority streams only
  if (hipStreamCreateWithFlags(&c->sA, hipStreamNonBlocking) != hipSuccess ||
      hipStreamCreateWithFlags(&c->sB, hipStreamNonBlocking) != hipSuccess)
    return die(TKV_EDEVICE, "tkv_create: hipStreamCreate failed");
  bool evok = hipEventCreateWithFlags(&c->ev_plan, hipEventDisableTiming) == hipSuccess;
  for (int i = 0; i < RING && evok; ++i) evok = hipEventCreateWithFlags(&c->ev_piece[i], hipEventDisableTiming) == hipSuccess;
  for (int l = 0; l < L && evok; ++l) evok = hipEventCreateWithFlags(&c->ev_ready[l], hipEventDisableTiming) == hipSuccess;
  for (int f = 0; f < 2 && evok && c->streamed; ++f)
    evok = hipEventCreateWithFlags(&c->ev_filled[f], hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&c->ev_free[f], hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&c->ev_gath[f], hipEventDisableTiming) == hipSuccess;
  for (int i = 0; i < RING && evok && c->streamed; ++i)
    evok = hipEventCreateWithFlags(&c->ev_h2d[i], hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&c->ev_scat[i], hipEventDisableTiming) == hipSuccess;
  if (c->streamed && hipStreamCreateWithFlags(&c->sC, hipStreamNonBlocking) != hipSuccess)
    return die(TKV_EDEVICE, "tkv_create: hipStreamCreate failed");
  if (!evok) return die(TKV_EDEVICE, "tkv_create: hipEventCreate failed");
  if (launch_init_state(v, nullptr) != hipSuccess || hipStreamSynchronize(nullptr) != hipSuccess)
    return die(TKV_EDEVICE, "tkv_create: state initialisation failed");
  *out = c;
  return TKV_OK;
}

void tkv_destroy(tkv_cache* c) {
  if (!c) return;
  (void)hipDeviceSynchronize();
  if (c->sA) (void)hipStreamDestroy(c->sA);
  if (c->sB) (void)hipStreamDestroy(c->sB);
  if (c->sC) (void)hipStreamDestroy(c->sC);
  for (auto e : c->ev_h2d) if (e) (void)hipEventDestroy(e);
  for (auto e : c->ev_scat) if (e) (void)hipEventDestroy(e);
  if (c->ev_plan) (void)hipEventDestroy(c->ev_plan);
  for (auto e : c->ev_piece) if (e) (void)hipEventDestroy(e);
  for (auto e : c->ev_ready) if (e) (void)hipEventDestroy(e);
  for (auto e : c->ev_filled) if (e) (void)hipEventDestroy(e);
  for (auto e : c->ev_free) if (e) (void)hipEventDestroy(e);
  for (auto e : c->ev_gath) if (e) (void)hipEventDestroy(e);
  for (auto& p : c->copy_events) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
  for (auto& p : c->prof_events) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
  for (auto& p : c->step_events) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
  for (void* p : c->dev_allocs) { if (c->cfg.dev_free) c->cfg.dev_free(p, c->cfg.alloc_ctx); else (void)hipFree(p); }
  for (void* p : c->pin_allocs) { if (c->cfg.pin_free) c->cfg.pin_free(p, c->cfg.alloc_ctx); else (void)hipHostFree(p); }
  delete c;
}

int32_t tkv_layer_length(const tkv_cache* c, int32_t layer) {
  if (!c || layer < 0 || layer >= c->cfg.n_layers) return -1;
  return c->len[layer];
}

tkv_status tkv_append(tkv_cache* c, int32_t layer, const void* k, const void* v, int32_t n_new, void* hip_stream) {
  if (!c) return TKV_EINVAL;
  if (layer < 0 || layer >= c->cfg.n_layers || !k || !v || n_new < 1) return fail(c, TKV_EINVAL, "tkv_append: bad argument");
  if (c->plan_pending) return fail(c, TKV_ESTATE, "tkv_append: a tier plan is pending; call tkv_migrate first");
  const int pos0 = c->len[layer];
  if ((int64_t)pos0 + n_new > c->cfg.max_tokens) return fail(c, TKV_ECAPACITY, "tkv_append: %d + %d exceeds max_tokens %d", pos0, n_new, c->cfg.max_tokens);
  bool assign = false;
  if (pos0 + n_new > c->n_assigned) {
    if (pos0 != c->n_assigned) return fail(c, TKV_ESTATE, "tkv_append: layer %d at length %d would overlap the assigned range %d", layer, pos0, c->n_assigned);
    for (int b = 0; b < c->cfg.batch; ++b)
      if (c->free0[b] < n_new) return fail(c, TKV_ECAPACITY, "tkv_append: HBM pool of sequence %d has %d free slots, need %d", b, c->free0[b], n_new);
    assign = true;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  HIPCHK(c, launch_append(c->dv, layer, k, v, pos0, n_new, assign, st));
  if (assign) {
    for (int b = 0; b < c->cfg.batch; ++b) { c->free0[b] -= n_new; c->nF[b] += n_new; }
    c->ntier[0] += (int64_t)n_new * c->cfg.batch;
    c->n_assigned += n_new;
  }
  c->len[layer] = pos0 + n_new;
  return TKV_OK;
}

// Most query tokens of a chunk that one launch serves; longer chunks go in groups.  16-bit rows: as many as fit the
// 16 columns of a workgroup's accumulators beside the group's heads (the cache is read once for all of them); binary32
// rows: one workgroup set per token along the grid.
static int chunk_tokens_per_launch(const tkv_cache* c) {
  return c->es == 2 ? attn_cols_per_launch(2, c->G) : 8;
}

// Scratch for launches that serve several query tokens per sequence: logits and split partials per (sequence, query).
// Allocated on the first such call, for as many queries as one launch takes, and kept until the cache is destroyed.
static tkv_status chunk_scratch(tkv_cache* c) {
  if (c->xs_chunk) return TKV_OK;
  const DevView& v = c->dv;
  const size_t nb = (size_t)v.B * chunk_tokens_per_launch(c);
  float *x = nullptr, *ml = nullptr, *po = nullptr;
  if (!dalloc(c, x, nb * v.Hq * c->xs_stride) || !dalloc(c, ml, nb * v.Hkv * c->S_alloc * 2 * c->G) ||
      !dalloc(c, po, nb * v.Hkv * c->S_alloc * c->G * v.D))
    return fail(c, TKV_ENOMEM, "tkv_attend_and_score_chunk: no device memory for the scratch of %d query tokens per launch", chunk_tokens_per_launch(c));
  c->xs_chunk = x; c->ml_chunk = ml; c->po_chunk = po;
  return TKV_OK;
}

// m query tokens per sequence (m = 1: a decode step's one) against one layer.  trim: entries at the end of list F that
// the last of the m queries leaves out (later tokens of a chunk); query j of the m leaves m - 1 - j more out.  q_bs /
// o_bs: query heads between consecutive sequences in q / out, the m queries of a sequence being Hq heads apart; last:
// the layer's last call of this step (the streamed frame is released and refilled, queued transfers are pumped).
// noalloc: the scratch of the call lives in the library's fixed device array, and nothing on the way may allocate
// (no event pools, no queued transfers are issued).
static tkv_status attend_one(tkv_cache* c, int32_t layer, const void* q, void* out, int trim, int q_bs, int o_bs, bool last,
                             hipStream_t st, bool noalloc = false, int m = 1) {
  const DevView& v = c->dv;
  if (m > 1) {
    if (c->streamed || noalloc || m > chunk_tokens_per_launch(c)) return fail(c, TKV_EINVAL, "attend_one: %d queries per launch not possible here", m);
    tkv_status cs = chunk_scratch(c);
    if (cs != TKV_OK) return cs;
  }
  bool use_old = false;
  const int fr = layer & 1;
  if (c->streamed) {
    // the layer's T1 rows must be in its frame (normally the fill was issued two layers ago)
    bool any = false;
    for (int b = 0; b < v.B; ++b) any = any || c->nS[b] > 0;
    if (any) {
      if (c->frame_layer[fr] != layer) { tkv_status fs = issue_fill(c, layer, fr); if (fs != TKV_OK) return fs; }
      HIPCHK(c, hipStreamWaitEvent(st, c->ev_filled[fr], 0));
      c->st.attend_waits++;
    }
  } else if (c->layer_wait[layer]) {
    if (c->cfg.prefetch_mode == TKV_PREFETCH_WAIT) {
      while (!noalloc && !c->layer_enq[layer] && c->jobs_next < c->jobs.size()) {
        tkv_status ps = pump_transfers(c, 1);
        if (ps != TKV_OK) return ps;
      }
      if (!c->layer_enq[layer]) return fail(c, TKV_ESTATE, "tkv_attend_and_score: the transfers of layer %d have not been queued", layer);
      HIPCHK(c, hipStreamWaitEvent(st, c->ev_ready[layer], 0));
      c->layer_wait[layer] = 0;
      c->st.attend_waits++;
    } else {
      // a layer whose pieces are still queued on the host keeps its old slots, like one whose copies are in flight
      hipError_t e = c->layer_enq[layer] ? hipEventQuery(c->ev_ready[layer]) : hipErrorNotReady;
      if (e == hipSuccess) c->layer_wait[layer] = 0;
      else if (e == hipErrorNotReady) { use_old = true; c->st.lazy_old_reads++; }
      else return fail(c, TKV_EDEVICE, "hipEventQuery failed: %s", hipGetErrorString(e));
    }
  }
  auto tiles = [](int n) { return (n + TOK_PER_BLOCK - 1) / TOK_PER_BLOCK; };
  int n_tiles = 1, n_tiles_s = 0;
  for (int b = 0; b < v.B; ++b) {
    n_tiles = std::max(n_tiles, tiles(c->nF[b] - trim) + tiles(c->nQ[b]) + tiles(c->nS[b]));
    n_tiles_s = std::max(n_tiles_s, tiles(c->nS[b]));
  }
  if (n_tiles * TOK_PER_BLOCK > c->xs_stride) return fail(c, TKV_ESTATE, "tkv_attend_and_score: internal tile count %d exceeds the scratch", n_tiles);
  // no more workgroups per pair than there are tiles for their waves
  const int nw = attn_waves_per_group(v.D, c->es, c->G, m);
  const int S = std::max(1, std::min(c->S_alloc, (n_tiles - n_tiles_s + nw - 1) / nw));
  const int S2 = n_tiles_s > 0 ? std::max(1, std::min(c->S_alloc, (n_tiles_s + nw - 1) / nw)) : 0;
  AttnArgs a{};
  const size_t lrows = (size_t)layer * v.B * v.Hkv;
  a.fpK = v.fpK + lrows * v.capP * v.D * v.es; a.fpV = v.fpV + lrows * v.capP * v.D * v.es;
  a.c2K = v.c2K + lrows * v.cap2 * v.cb; a.c2V = v.c2V + lrows * v.cap2 * v.cb;
  a.s2K = v.s2K + lrows * v.cap2 * v.sb; a.s2V = v.s2V + lrows * v.cap2 * v.sb;
  a.q = q; a.out = out;
  a.f_loc = use_old ? v.f_loc_old : v.f_loc; a.f_pos = v.f_pos; a.q_loc = v.q_loc; a.q_pos = v.q_pos;
  a.vnorm = v.vnorm ? v.vnorm + lrows * v.Nmax : nullptr;
  a.red = v.red ? v.red + lrows * v.Nmax : nullptr;
  a.red_w = c->cfg.redundancy_weight > 0.f ? c->cfg.redundancy_weight : 1.0f;
  a.cnt = v.cnt; a.score = v.score; a.xs = c->xs; a.part_ml = c->part_ml; a.part_o = c->part_o;
  if (m > 1) { a.xs = c->xs_chunk; a.part_ml = c->ml_chunk; a.part_o = c->po_chunk; }
  if (noalloc) {
    // the same three arrays, carved out of the fixed scratch array (256-byte aligned each)
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t xs_b = up((size_t)v.B * v.Hq * c->xs_stride * sizeof(float));
    const size_t ml_b = up((size_t)v.B * v.Hkv * c->S_alloc * 2 * c->G * sizeof(float));
    const size_t po_b = up((size_t)v.B * v.Hkv * c->S_alloc * c->G * v.D * sizeof(float));
    if (xs_b + ml_b + po_b > NOALLOC_SCRATCH_BYTES)
      return fail(c, TKV_ECAPACITY, "tkv_attend_and_score_noalloc: this cache needs %zu bytes of scratch per call, the fixed array holds %zu",
                  xs_b + ml_b + po_b, NOALLOC_SCRATCH_BYTES);
    a.xs = (float*)c->static_scratch; a.part_ml = (float*)(c->static_scratch + xs_b); a.part_o = (float*)(c->static_scratch + xs_b + ml_b);
  }
  a.q_es = c->es;
  if (v.B <= ATTN_ARG_SEQS)
    for (int b = 0; b < v.B; ++b) {
      a.nF[b] = c->nF[b] - trim; a.nQ[b] = c->nQ[b];
      a.nWq[b] = attn_q_waves(S * nw, tiles(c->nF[b] - trim), tiles(c->nQ[b]));
    }
  a.B = v.B; a.Hq = v.Hq; a.Hkv = v.Hkv; a.Nmax = v.Nmax; a.capF = v.capP; a.cap2 = v.cap2;
  a.S = S; a.S_total = S + S2; a.s0 = 0; a.second = 0; a.s_pos = c->streamed ? v.s_pos : nullptr; a.n_tiles = n_tiles; a.xs_stride = c->xs_stride; a.cb = v.cb; a.sb = v.sb; a.t2fmt = v.t2fmt; a.out_kind = c->cfg.out_dtype;
  a.softmax_scale = c->softmax_scale; a.score_scale = c->score_scale;
  a.q_bs = q_bs; a.o_bs = o_bs; a.trim = trim;
  if (c->es == 2) { a.n_q = 1; a.cq = m; } else { a.n_q = m; a.cq = 1; }   // 16-bit rows: the tokens as columns of one workgroup
  EvPair* pe = nullptr;
  EvPair* pe2 = nullptr;
  EvPair* pf = nullptr;
  if ((c->cfg.profile & 1) && !noalloc) {
    const size_t i0 = c->prof_used;
    if (!next_pair(c->prof_events, c->prof_used) || (S2 > 0 && !next_pair(c->prof_events, c->prof_used)) ||
        !next_pair(c->prof_events, c->prof_used))
      return fail(c, TKV_EDEVICE, "hipEventCreate failed");
    pe = &c->prof_events[i0];          // taken after the pool has stopped growing
    pe->dir = 0;
    if (S2 > 0) { pe2 = &c->prof_events[i0 + 1]; pe2->dir = 2; }
    pf = &c->prof_events[c->prof_used - 1];
    pf->dir = 3; pf->bytes = (int64_t)i0;   // index of the call's first kernel
  }
  HIPCHK(c, launch_attn_tiered(a, v.D, c->G, c->kt, st, pe ? pe->a : nullptr, pe ? pe->b : nullptr));
  if (S2 > 0) {
    // streamed T1: the same kernel over the T1 list, rows in the frame; its splits follow the first launch's
    AttnArgs a2 = a;
    a2.fpK = c->frameK[fr]; a2.fpV = c->frameV[fr]; a2.capF = v.cap1;
    a2.f_loc = v.s_loc; a2.f_pos = v.s_pos;
    a2.S = S2; a2.s0 = S; a2.second = 1;
    HIPCHK(c, launch_attn_tiered(a2, v.D, c->G, c->kt, st, pe2 ? pe2->a : nullptr, pe2 ? pe2->b : nullptr));
  }
  if (m > 1) HIPCHK(c, launch_attn_finish_chunk(a, v.D, c->G, st));
  else HIPCHK(c, launch_attn_finish(a, v.D, c->G, st, pf ? pf->a : nullptr, pf ? pf->b : nullptr));
  if (!last || noalloc) return TKV_OK;
  if (c->streamed && S2 > 0) {
    HIPCHK(c, hipEventRecord(c->ev_free[fr], st));
    c->frame_used[fr] = true;
    // refill this frame for the layer that uses it next (two layers on, or the next step's first layers)
    const int L = v.L;
    const int nxt = layer + 2 < L ? layer + 2 : fr;
    if (nxt < L && nxt != layer) { tkv_status fs = issue_fill(c, nxt, fr); if (fs != TKV_OK) return fs; }
    return TKV_OK;
  }
  // lazy mode spreads the issue of a re-tiering event's copies over the following attention calls, one layer each,
  // so the compute stream is never left empty while the host queues them
  if (c->jobs_next < c->jobs.size()) return pump_transfers(c, 1);
  return TKV_OK;
}

tkv_status tkv_attend_and_score(tkv_cache* c, int32_t layer, const void* q, void* out, void* hip_stream) {
  if (!c) return TKV_EINVAL;
  if (layer < 0 || layer >= c->cfg.n_layers || !q || !out) return fail(c, TKV_EINVAL, "tkv_attend_and_score: bad argument");
  if (c->len[layer] == 0) return fail(c, TKV_ESTATE, "tkv_attend_and_score: layer %d is empty", layer);
  if (c->len[layer] != c->n_assigned) return fail(c, TKV_ESTATE, "tkv_attend_and_score: layer %d has %d tokens, %d are assigned; append first", layer, c->len[layer], c->n_assigned);
  return attend_one(c, layer, q, out, 0, c->dv.Hq, c->dv.Hq, true, (hipStream_t)hip_stream);
}

tkv_status tkv_attend_and_score_noalloc(tkv_cache* c, int32_t layer, const void* q, void* out, void* hip_stream) {
  if (!c) return TKV_EINVAL;
  if (layer < 0 || layer >= c->cfg.n_layers || !q || !out) return fail(c, TKV_EINVAL, "tkv_attend_and_score_noalloc: bad argument");
  if (c->streamed) return fail(c, TKV_EINVAL, "tkv_attend_and_score_noalloc: not available with TKV_PREFETCH_STREAM (its frame refills take events from a growing pool)");
  if (c->len[layer] == 0) return fail(c, TKV_ESTATE, "tkv_attend_and_score_noalloc: layer %d is empty", layer);
  if (c->len[layer] != c->n_assigned) return fail(c, TKV_ESTATE, "tkv_attend_and_score_noalloc: layer %d has %d tokens, %d are assigned; append first", layer, c->len[layer], c->n_assigned);
  return attend_one(c, layer, q, out, 0, c->dv.Hq, c->dv.Hq, true, (hipStream_t)hip_stream, true);
}

tkv_status tkv_attend_and_score_chunk(tkv_cache* c, int32_t layer, const void* q, void* out, int32_t n_q, void* hip_stream) {
  if (!c) return TKV_EINVAL;
  if (layer < 0 || layer >= c->cfg.n_layers || !q || !out || n_q < 1) return fail(c, TKV_EINVAL, "tkv_attend_and_score_chunk: bad argument");
  if (c->len[layer] == 0) return fail(c, TKV_ESTATE, "tkv_attend_and_score_chunk: layer %d is empty", layer);
  if (c->len[layer] != c->n_assigned) return fail(c, TKV_ESTATE, "tkv_attend_and_score_chunk: layer %d has %d tokens, %d are assigned; append first", layer, c->len[layer], c->n_assigned);
  // the chunk's positions must be the tail of list F: appended since the last plan was applied, so still in T0
  if (n_q > c->n_assigned - c->n_at_plan)
    return fail(c, TKV_ESTATE, "tkv_attend_and_score_chunk: %d query tokens, but only %d positions were appended since the last tkv_migrate", n_q, c->n_assigned - c->n_at_plan);
  const DevView& v = c->dv;
  const size_t q_tok = (size_t)v.Hq * v.D * c->es, o_tok = (size_t)v.Hq * v.D * (c->cfg.out_dtype == TKV_F32 ? 4 : 2);
  // The chunk's tokens go in groups of as many as one launch takes (16-bit rows: the cache is read once per group).
  // The streamed mode, whose frame serves one launch pair at a time, takes the tokens one by one.
  const int per = c->streamed ? 1 : chunk_tokens_per_launch(c);
  for (int j = 0; j < n_q; j += per) {
    const int m = std::min(per, n_q - j);
    tkv_status s = attend_one(c, layer, (const char*)q + j * q_tok, (char*)out + j * o_tok, n_q - j - m, n_q * v.Hq, n_q * v.Hq,
                              j + m == n_q, (hipStream_t)hip_stream, false, m);
    if (s != TKV_OK) return s;
  }
  return TKV_OK;
}

tkv_status tkv_decode_step(tkv_cache* c, const void* k_all, const void* v_all, const void* q_all, void* out_all,
                           void* hip_stream) {
  if (!c) return TKV_EINVAL;
  if (!k_all || !v_all || !q_all || !out_all) return fail(c, TKV_EINVAL, "tkv_decode_step: NULL argument");
  const DevView& v = c->dv;
  const size_t kv_stride = (size_t)v.B * v.Hkv * v.D * v.es;
  const size_t q_stride = (size_t)v.B * v.Hq * v.D * v.es;
  const size_t o_stride = (size_t)v.B * v.Hq * v.D * (c->cfg.out_dtype == TKV_F32 ? 4 : 2);
  // all layers are at the same length here, so the new token's rows of every layer go in with one launch
  const int n = common_length(c);
  if (n >= 0 && n == c->n_assigned && !c->plan_pending) {
    if (n + 1 > c->cfg.max_tokens) return fail(c, TKV_ECAPACITY, "tkv_decode_step: %d + 1 exceeds max_tokens %d", n, c->cfg.max_tokens);
    for (int b = 0; b < v.B; ++b)
      if (c->free0[b] < 1) return fail(c, TKV_ECAPACITY, "tkv_decode_step: HBM pool of sequence %d is full", b);
    EvPair* se = nullptr;
    if (c->cfg.profile & 2) {
      se = next_pair(c->step_events, c->step_used);
      if (!se) return fail(c, TKV_EDEVICE, "hipEventCreate failed");
      HIPCHK(c, hipEventRecord(se->a, (hipStream_t)hip_stream));
    }
    HIPCHK(c, launch_append_step(v, k_all, v_all, n, (hipStream_t)hip_stream));
    for (int b = 0; b < v.B; ++b) { c->free0[b] -= 1; c->nF[b] += 1; }
    c->ntier[0] += v.B;
    c->n_assigned += 1;
    for (int l = 0; l < v.L; ++l) c->len[l] = n + 1;
    for (int l = 0; l < v.L; ++l) {
      tkv_status s = tkv_attend_and_score(c, l, (const char*)q_all + l * q_stride, (char*)out_all + l * o_stride, hip_stream);
      if (s != TKV_OK) return s;
    }
    if (se) HIPCHK(c, hipEventRecord(se->b, (hipStream_t)hip_stream));
    return TKV_OK;
  }
  for (int l = 0; l < v.L; ++l) {
    tkv_status s = tkv_append(c, l, (const char*)k_all + l * kv_stride, (const char*)v_all + l * kv_stride, 1, hip_stream);
    if (s != TKV_OK) return s;
    s = tkv_attend_and_score(c, l, (const char*)q_all + l * q_stride, (char*)out_all + l * o_stride, hip_stream);
    if (s != TKV_OK) return s;
  }
  return TKV_OK;
}

tkv_status tkv_classify(tkv_cache* c, const tkv_policy* policy, void* hip_stream) {
  if (!c) return TKV_EINVAL;
  if (!policy_ok(policy)) return fail(c, TKV_EINVAL, "tkv_classify: policy fractions must sum to 1000000 ppm and count_rule be 0 or 1");
  const int n = common_length(c);
  if (n < 0 || n != c->n_assigned) return fail(c, TKV_ESTATE, "tkv_classify: layers differ in length");
  if (n == 0) return fail(c, TKV_ESTATE, "tkv_classify: cache is empty");
  const auto t0 = std::chrono::steady_clock::now();
  hipStream_t st = (hipStream_t)hip_stream;
  const uint32_t ppm[5] = {policy->f_t0_ppm, policy->f_t1_ppm, policy->f_t2_ppm, policy->f_t3_ppm, policy->count_rule};
  HIPCHK(c, launch_classify(c->dv, n, ppm, st));
  c->plan_pending = true;
  c->st.n_classify++;
  c->st.classify_ms += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
  return TKV_OK;
}

tkv_status tkv_migrate(tkv_cache* c, void* hip_stream) {
  if (!c) return TKV_EINVAL;
  if (!c->plan_pending) return fail(c, TKV_ESTATE, "tkv_migrate: no pending plan");
  const int n = common_length(c);
  if (n < 0 || n != c->n_assigned) return fail(c, TKV_ESTATE, "tkv_migrate: layers differ in length");
  const auto t0 = std::chrono::steady_clock::now();
  hipStream_t st = (hipStream_t)hip_stream;
  DevView& v = c->dv;
  const int B = v.B, L = v.L;
  // the previous migrate's transfers must have landed before its HBM slots are recycled
  tkv_status s = drain_transfers(c);
  if (s != TKV_OK) return s;
  int64_t total_new_t1 = 0;
  int max10 = 0, maxq = 0, maxd = 0;
  for (int pass = 0;; ++pass) {
  HIPCHK(c, launch_plan_count(v, n, st));
  HIPCHK(c, hipMemcpyAsync(c->pin_cnt, v.cnt, (size_t)B * CNT_N * sizeof(int), hipMemcpyDeviceToHost, st));
  HIPCHK(c, hipStreamSynchronize(st));
  total_new_t1 = 0; max10 = maxq = maxd = 0;
  int64_t live1 = 0, enter1 = 0;
  for (int b = 0; b < B; ++b) {
    const int* k = c->pin_cnt + b * CNT_N;
    if (k[C_BAD]) return fail(c, TKV_ESTATE, "tkv_migrate: the plan moves %d position(s) of sequence %d out of T3 or names an invalid tier", k[C_BAD], b);
    const int e0 = k[C_M10] + k[C_M20] + k[C_M21], e1 = k[C_M01] + k[C_M21], e2 = k[C_M02] + k[C_M12];
    if (e0 > k[C_FREE0] + k[C_PEND]) return fail(c, TKV_ECAPACITY, "tkv_migrate: HBM pool of sequence %d: %d rows enter, %d slots free", b, e0, k[C_FREE0] + k[C_PEND]);
    if (e1 > k[C_FREE1]) return fail(c, TKV_ECAPACITY, "tkv_migrate: staging buffer of sequence %d: %d rows enter, %d slots free", b, e1, k[C_FREE1]);
    if (e2 > k[C_FREE2]) return fail(c, TKV_ECAPACITY, "tkv_migrate: compressed pool of sequence %d: %d rows enter, %d slots free", b, e2, k[C_FREE2]);
    c->pin_base[b] = (int)(c->host_next + total_new_t1);
    total_new_t1 += e1 - k[C_M01R];              // rows that return to T1 with a valid host copy are not transferred
    live1 += k[C_N1]; enter1 += e1;
    max10 = std::max(max10, k[C_MCOPY]); maxq = std::max(maxq, e2); maxd = std::max(maxd, k[C_M20] + k[C_M21]);
  }
  if (c->host_next + total_new_t1 <= c->host_rows) break;
  // The store hands out rows in order and has too few left.  Packed, it needs the rows T1 holds now plus every row
  // that enters (none of which keeps a host copy across the rewrite); if that fits, rewrite it and count again.
  if (pass > 0 || live1 + enter1 > c->host_rows)
    return fail(c, TKV_ECAPACITY, "tkv_migrate: pinned T1 store: %lld rows in T1, %lld enter, capacity %lld",
                (long long)live1, (long long)enter1, (long long)c->host_rows);
  tkv_status rs = rehome_store(c, n, st);
  if (rs != TKV_OK) return rs;
  }
  HIPCHK(c, hipMemcpyAsync(c->d_host_base, c->pin_base, (size_t)B * sizeof(int), hipMemcpyHostToDevice, st));
  v.event_base = (int)c->host_next;
  HIPCHK(c, launch_plan_commit(v, n, st));
  if (!c->streamed) {
    HIPCHK(c, launch_moves(v, max10, maxq, maxd, st));
  } else {
    // Rows that leave T1 for T0 or T2 are read from a frame, layer by layer, each after a fill from the pinned store
    // (the table of host rows still names them; they are struck from it afterwards).  Rows that come out of T2 and
    // rows that only move inside HBM do not need the frames.
    HIPCHK(c, launch_decode_moves(v, maxd, st));
    int64_t from_t1 = 0, leaving = 0, live1 = 0, new_total = 0;
    int max_leaving = 0;
    for (int b = 0; b < B; ++b) {
      const int* k = c->pin_cnt + b * CNT_N;
      from_t1 += k[C_M10] + k[C_M12];
      leaving += k[C_M10] + k[C_M12] + k[C_M13];
      live1 += k[C_N1];
      max_leaving = std::max(max_leaving, k[C_M10] + k[C_M12] + k[C_M13]);
      c->pin_base[B + b] = (int)new_total; new_total += k[C_P1];
    }
    c->frame_layer[0] = c->frame_layer[1] = -1;
    // Rows of the pinned store whose position is not in T1 any more cross the link at every later step for nothing.
    // Rewriting the store packed costs about one copy of T1 (device to host, beside this migrate's fills); it pays
    // when the stale rows, over the steps until the next plan (taken to be as many as since the last one), would
    // cost more.
    const int64_t stale_after = (c->host_next - live1) + leaving;
    const int64_t steps_between = std::max(1, n - c->n_at_plan);
    if (max_leaving > 0 && stale_after * steps_between >= new_total) {
      // The store is rewritten while the plan is applied: every layer passes through a frame (the rows that leave
      // T1 for T0 or T2 are read from it); behind the movers the offload stream gathers the layer's new T1 set (rows
      // that stay, from the frame; rows that enter, from their HBM slots) in the new order and copies it over the
      // layer's part of the store, which the fill has finished reading by then.
      HIPCHK(c, hipMemcpyAsync(c->d_base2, c->pin_base + B, (size_t)B * sizeof(int), hipMemcpyHostToDevice, st));
      HIPCHK(c, launch_repack_number(v, n, c->d_base2, c->g2_seq, c->g2_src, c->hloc2, st));
      HIPCHK(c, hipEventRecord(c->ev_plan, st));
      HIPCHK(c, hipStreamWaitEvent(c->sB, c->ev_plan, 0));
      HIPCHK(c, hipStreamWaitEvent(c->sA, c->ev_plan, 0));
      const size_t slot_bytes = c->bounce_bytes / RING;
      const int64_t piece_rows = std::max<int64_t>(1, (int64_t)(slot_bytes / c->tok_bytes));
      int piece = 0;
      for (int l = 0; l < L; ++l) {
        const int f = l & 1;
        tkv_status fs = issue_fill(c, l, f);
        if (fs != TKV_OK) return fs;
        DevView vv = v;
        vv.frK = c->frameK[f]; vv.frV = c->frameV[f];
        if (from_t1 > 0) {
          HIPCHK(c, hipStreamWaitEvent(st, c->ev_filled[f], 0));
          HIPCHK(c, launch_moves_layer(vv, l, max10, maxq, st));
        }
        HIPCHK(c, hipStreamWaitEvent(c->sA, c->ev_filled[f], 0));
        DevView vg = vv;
        vg.g_seq = c->g2_seq; vg.g_src = c->g2_src;
        EvPair* ed = next_pair(c->copy_events, c->copy_events_used);
        if (!ed) return fail(c, TKV_EDEVICE, "hipEventCreate failed");
        ed->dir = 0; ed->bytes = 0;
        HIPCHK(c, hipEventRecord(ed->a, c->sA));
        for (int64_t r0 = 0; r0 < new_total; r0 += piece_rows, ++piece) {
          const int nrows = (int)std::min<int64_t>(piece_rows, new_total - r0);
          const size_t bytes = (size_t)nrows * c->tok_bytes;
          char* ba = c->bounceA + (size_t)(piece % RING) * slot_bytes;   // one stream: a ring slot is refilled after its copy
          HIPCHK(c, launch_gather(vg, l, (int)r0, nrows, ba, c->sA));
          if (r0 + piece_rows >= new_total) HIPCHK(c, hipEventRecord(c->ev_gath[f], c->sA));   // the frame has been read
          HIPCHK(c, hipMemcpyAsync(c->hstore + ((size_t)l * c->host_rows + (size_t)r0) * c->tok_bytes, ba, bytes,
                                   hipMemcpyDeviceToHost, c->sA));
          c->st.d2h_bytes += (int64_t)bytes; c->st.d2h_copies++;
        }
        if (new_total == 0) HIPCHK(c, hipEventRecord(c->ev_gath[f], c->sA));
        HIPCHK(c, hipEventRecord(ed->b, c->sA));
        HIPCHK(c, hipEventRecord(c->ev_ready[l], c->sA));       // the layer's next fill waits for its part of the store
        c->layer_wait[l] = 1; c->layer_enq[l] = 1;
        HIPCHK(c, hipStreamWaitEvent(st, c->ev_gath[f], 0));
        HIPCHK(c, hipEventRecord(c->ev_free[f], st));
        c->frame_used[f] = true;
      }
      if (from_t1 == 0) HIPCHK(c, launch_moves(v, max10, maxq, 0, st));
      // the new numbering takes over: the fills above went by the old table, the next ones go by the new one
      for (int f = 0; f < 2; ++f) HIPCHK(c, hipStreamWaitEvent(st, c->ev_filled[f], 0));
      HIPCHK(c, launch_repack_apply(v, n, c->hloc2, st));
      HIPCHK(c, launch_rebuild_htable(v, n, (int)c->host_rows, st));
      for (int f = 0; f < 2; ++f) HIPCHK(c, hipEventRecord(c->ev_free[f], st));
      c->frame_layer[0] = c->frame_layer[1] = -1;
      c->host_next = new_total;
      c->transfers_in_flight = true;
      c->st.n_repack++;
      total_new_t1 = 0;                 // the rows that enter T1 went to the store with the rest
    } else if (from_t1 == 0) {
      HIPCHK(c, launch_moves(v, max10, maxq, 0, st));
      HIPCHK(c, launch_clear_host_rows(v, max_leaving, st));
    } else {
      // the rows that leave T1 for T0 or T2 are read from a frame, layer by layer; the table of host rows still names
      // them and they are struck from it afterwards
      HIPCHK(c, hipEventRecord(c->ev_plan, st));
      HIPCHK(c, hipStreamWaitEvent(c->sB, c->ev_plan, 0));
      for (int l = 0; l < L; ++l) {
        const int f = l & 1;
        tkv_status fs = issue_fill(c, l, f);
        if (fs != TKV_OK) return fs;
        HIPCHK(c, hipStreamWaitEvent(st, c->ev_filled[f], 0));
        DevView vv = v;
        vv.frK = c->frameK[f]; vv.frV = c->frameV[f];
        HIPCHK(c, launch_moves_layer(vv, l, max10, maxq, st));
        HIPCHK(c, hipEventRecord(c->ev_free[f], st));
        c->frame_used[f] = true;
      }
      c->frame_layer[0] = c->frame_layer[1] = -1;   // the frames hold the rows of the old plan
      HIPCHK(c, launch_clear_host_rows(v, max_leaving, st));
    }
  }
  // host mirrors of what plan_commit leaves on the device
  for (int t = 0; t < 4; ++t) c->ntier[t] = 0;
  for (int b = 0; b < B; ++b) {
    const int* k = c->pin_cnt + b * CNT_N;
    c->nF[b] = c->streamed ? k[C_P0] : k[C_P0] + k[C_P1]; c->nQ[b] = k[C_P2]; c->nS[b] = c->streamed ? k[C_P1] : 0;
    for (int t = 0; t < 4; ++t) c->ntier[t] += k[C_P0 + t];
    const int e0 = k[C_M10] + k[C_M20] + k[C_M21], e1 = k[C_M01] + k[C_M21], e2 = k[C_M02] + k[C_M12];
    c->free0[b] = k[C_FREE0] + k[C_PEND] - e0 + k[C_M02] + k[C_M03] + k[C_M01R];
    c->pend[b] = e1 - k[C_M01R];
    c->free1[b] = k[C_FREE1] - e1 + k[C_M10] + k[C_M12] + k[C_M13];
    c->free2[b] = k[C_FREE2] - e2 + k[C_M20] + k[C_M21] + k[C_M23];
  }
  if (total_new_t1 > 0) {
    // offload stream: gather -> D2H into the pinned store; prefetch stream: H2D -> scatter into the staging slots
    HIPCHK(c, hipEventRecord(c->ev_plan, st));
    HIPCHK(c, hipStreamWaitEvent(c->sA, c->ev_plan, 0));
    HIPCHK(c, hipStreamWaitEvent(c->sB, c->ev_plan, 0));
    const size_t slot_bytes = c->bounce_bytes / RING;
    const int64_t piece_rows = std::max<int64_t>(1, (int64_t)(slot_bytes / c->tok_bytes));
    int piece = 0;
    c->jobs.clear(); c->jobs_next = 0;
    // when a layer's rows fill only part of a bounce piece, several layers share one (one strided copy each way
    // instead of one per layer: the copies disturb the attention kernels per copy, not per byte)
    const int group = total_new_t1 <= piece_rows ? (int)std::min<int64_t>(L, piece_rows / total_new_t1) : 1;
    for (int l = 0; l < L; l += group) {
      const int nl = std::min(group, L - l);
      for (int64_t r0 = 0; r0 < total_new_t1; r0 += piece_rows, ++piece) {
        const int nrows = (int)std::min<int64_t>(piece_rows, total_new_t1 - r0);
        c->jobs.push_back(XferJob{l, (int)r0, nrows, piece, c->host_next + r0, r0 + piece_rows >= total_new_t1, nl});
      }
      for (int li = 0; li < nl; ++li) { c->layer_wait[l + li] = 1; c->layer_enq[l + li] = 0; }
    }
    if (c->cfg.prefetch_mode != TKV_PREFETCH_LAZY) {
      tkv_status ps = pump_transfers(c, L);
      if (ps != TKV_OK) return ps;
    }
    c->transfers_in_flight = true;
    c->host_next += total_new_t1;
  }
  c->plan_pending = false;
  c->n_at_plan = n;
  c->st.n_migrate++;
  c->st.migrate_ms += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
  return TKV_OK;
}

tkv_status tkv_wait_prefetch(tkv_cache* c) {
  if (!c) return TKV_EINVAL;
  return drain_transfers(c);
}

// ---- inspection -------------------------------------------------------------------------------------------
static tkv_status sync_all(tkv_cache* c) {
  HIPCHK(c, hipDeviceSynchronize());
  return TKV_OK;
}

tkv_status tkv_get_scores(tkv_cache* c, float* host_out) {
  if (!c || !host_out) return c ? fail(c, TKV_EINVAL, "tkv_get_scores: NULL") : TKV_EINVAL;
  tkv_status s = sync_all(c); if (s) return s;
  HIPCHK(c, hipMemcpy(host_out, c->dv.score, (size_t)c->dv.B * c->dv.Nmax * sizeof(float), hipMemcpyDeviceToHost));
  return TKV_OK;
}
tkv_status tkv_set_scores(tkv_cache* c, const float* host_in) {
  if (!c || !host_in) return c ? fail(c, TKV_EINVAL, "tkv_set_scores: NULL") : TKV_EINVAL;
  const size_t n = (size_t)c->dv.B * c->dv.Nmax;
  for (size_t i = 0; i < n; ++i) if (!(host_in[i] >= 0.f) || std::signbit(host_in[i])) return fail(c, TKV_EINVAL, "tkv_set_scores: scores must be >= +0");
  tkv_status s = sync_all(c); if (s) return s;
  HIPCHK(c, hipMemcpy(c->dv.score, host_in, n * sizeof(float), hipMemcpyHostToDevice));
  return TKV_OK;
}
tkv_status tkv_get_tiers(tkv_cache* c, uint8_t* host_out) {
  if (!c || !host_out) return c ? fail(c, TKV_EINVAL, "tkv_get_tiers: NULL") : TKV_EINVAL;
  tkv_status s = sync_all(c); if (s) return s;
  HIPCHK(c, hipMemcpy(host_out, c->dv.tier, (size_t)c->dv.B * c->dv.Nmax, hipMemcpyDeviceToHost));
  return TKV_OK;
}
tkv_status tkv_get_pending_tiers(tkv_cache* c, uint8_t* host_out) {
  if (!c || !host_out) return c ? fail(c, TKV_EINVAL, "tkv_get_pending_tiers: NULL") : TKV_EINVAL;
  if (!c->plan_pending) return fail(c, TKV_ESTATE, "tkv_get_pending_tiers: no pending plan");
  tkv_status s = sync_all(c); if (s) return s;
  HIPCHK(c, hipMemcpy(host_out, c->dv.tier_new, (size_t)c->dv.B * c->dv.Nmax, hipMemcpyDeviceToHost));
  return TKV_OK;
}
tkv_status tkv_set_tiers(tkv_cache* c, const uint8_t* host_in) {
  if (!c || !host_in) return c ? fail(c, TKV_EINVAL, "tkv_set_tiers: NULL") : TKV_EINVAL;
  const int n = common_length(c);
  if (n < 0 || n != c->n_assigned) return fail(c, TKV_ESTATE, "tkv_set_tiers: layers differ in length");
  for (int b = 0; b < c->dv.B; ++b)
    for (int i = 0; i < n; ++i)
      if (host_in[(size_t)b * c->dv.Nmax + i] > 3) return fail(c, TKV_EINVAL, "tkv_set_tiers: tier > 3 at (%d, %d)", b, i);
  tkv_status s = sync_all(c); if (s) return s;
  HIPCHK(c, hipMemcpy(c->dv.tier_new, host_in, (size_t)c->dv.B * c->dv.Nmax, hipMemcpyHostToDevice));
  c->plan_pending = true;
  return TKV_OK;
}
tkv_status tkv_get_index_list(tkv_cache* c, int32_t tier, int32_t seq, int32_t* host_out, int32_t* count) {
  if (!c || !host_out || !count) return c ? fail(c, TKV_EINVAL, "tkv_get_index_list: NULL") : TKV_EINVAL;
  if (tier < 0 || tier > 3 || seq < 0 || seq >= c->dv.B) return fail(c, TKV_EINVAL, "tkv_get_index_list: bad tier or sequence");
  tkv_status s = sync_all(c); if (s) return s;
  int n = 0;
  HIPCHK(c, hipMemcpy(&n, c->dv.cnt + seq * CNT_N + C_N0 + tier, sizeof(int), hipMemcpyDeviceToHost));
  if (n < 0 || n > c->dv.Nmax) return fail(c, TKV_EDEVICE, "tkv_get_index_list: corrupt count %d", n);
  if (n) HIPCHK(c, hipMemcpy(host_out, c->dv.idx + ((size_t)tier * c->dv.B + seq) * c->dv.Nmax, (size_t)n * sizeof(int), hipMemcpyDeviceToHost));
  *count = n;
  return TKV_OK;
}

static tkv_status row_lookup(tkv_cache* c, const char* who, int32_t layer, int32_t seq, int32_t kvh, int32_t pos, int32_t which,
                             int* tier, int* loc, int* hloc) {
  const DevView& v = c->dv;
  if (layer < 0 || layer >= v.L || seq < 0 || seq >= v.B || kvh < 0 || kvh >= v.Hkv || pos < 0 || pos >= c->len[layer] ||
      pos >= c->n_assigned || which < 0 || which > 1)
    return fail(c, TKV_EINVAL, "%s: bad index", who);
  tkv_status s = sync_all(c); if (s) return s;
  uint8_t t8 = 0;
  const size_t o = (size_t)seq * v.Nmax + pos;
  HIPCHK(c, hipMemcpy(&t8, v.tier + o, 1, hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(loc, v.loc + o, sizeof(int), hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(hloc, v.hloc + o, sizeof(int), hipMemcpyDeviceToHost));
  *tier = t8;
  return TKV_OK;
}

tkv_status tkv_get_t2_row(tkv_cache* c, int32_t layer, int32_t seq, int32_t kv_head, int32_t pos, int32_t which,
                          void* host_codes, void* host_scales) {
  if (!c || !host_codes || !host_scales) return c ? fail(c, TKV_EINVAL, "tkv_get_t2_row: NULL") : TKV_EINVAL;
  int tier, loc, hloc;
  tkv_status s = row_lookup(c, "tkv_get_t2_row", layer, seq, kv_head, pos, which, &tier, &loc, &hloc);
  if (s) return s;
  const DevView& v = c->dv;
  if (tier != 2 || loc < 0 || loc >= v.cap2) return fail(c, TKV_ESTATE, "tkv_get_t2_row: position %d is in tier %d", pos, tier);
  const size_t r = (((size_t)layer * v.B + seq) * v.Hkv + kv_head) * v.cap2 + loc;
  HIPCHK(c, hipMemcpy(host_codes, (which ? v.c2V : v.c2K) + r * v.cb, v.cb, hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(host_scales, (which ? v.s2V : v.s2K) + r * v.sb, v.sb, hipMemcpyDeviceToHost));
  return TKV_OK;
}

tkv_status tkv_get_row(tkv_cache* c, int32_t layer, int32_t seq, int32_t kv_head, int32_t pos, int32_t which, void* host_out) {
  if (!c || !host_out) return c ? fail(c, TKV_EINVAL, "tkv_get_row: NULL") : TKV_EINVAL;
  int tier, loc, hloc;
  tkv_status s = row_lookup(c, "tkv_get_row", layer, seq, kv_head, pos, which, &tier, &loc, &hloc);
  if (s) return s;
  const DevView& v = c->dv;
  const size_t rb = (size_t)v.D * v.es;
  if (tier == 0) {
    if (loc < 0 || loc >= v.capF) return fail(c, TKV_EDEVICE, "tkv_get_row: corrupt slot %d", loc);
    const size_t off = ((((size_t)layer * v.B + seq) * v.Hkv + kv_head) * v.capP + loc) * rb;
    HIPCHK(c, hipMemcpy(host_out, (which ? v.fpV : v.fpK) + off, rb, hipMemcpyDeviceToHost));
    return TKV_OK;
  }
  if (tier == 1) {
    s = drain_transfers(c); if (s) return s;
    if (hloc < 0 || hloc >= c->host_rows) return fail(c, TKV_EDEVICE, "tkv_get_row: corrupt host row %d", hloc);
    const char* p = c->hstore + ((size_t)layer * c->host_rows + hloc) * c->tok_bytes + ((size_t)kv_head * 2 + which) * rb;
    memcpy(host_out, p, rb);
    return TKV_OK;
  }
  return fail(c, TKV_ESTATE, "tkv_get_row: position %d is in tier %d", pos, tier);
}

tkv_status tkv_probe_hbm_read(const void* device_buf, size_t bytes, int32_t iters, void* hip_stream, float* ms_per_pass) {
  if (!device_buf || bytes < 16 || iters < 1 || !ms_per_pass) return TKV_EINVAL;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    return TKV_EDEVICE;
  uint32_t* sink = (uint32_t*)scratch_on_device(dev);      // never written: the probe's condition does not hold for its data
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (!sink || hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return TKV_EDEVICE;
  hipStream_t st = (hipStream_t)hip_stream;
  double total = 0.0;
  tkv_status rc = TKV_OK;
  for (int i = 0; i < iters + 1 && rc == TKV_OK; ++i) {      // the first pass warms up and is not counted
    float ms = 0.f;
    if (launch_probe_read(device_buf, bytes, cus, sink, st, e0, e1) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
        hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = TKV_EDEVICE;
    if (i > 0) total += ms;
  }
  (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
  *ms_per_pass = (float)(total / iters);
  return rc;
}

tkv_status tkv_set_profile(tkv_cache* c, int32_t on) {
  if (!c) return TKV_EINVAL;
  c->cfg.profile = on & 3;
  return TKV_OK;
}

tkv_status tkv_get_stats(tkv_cache* c, tkv_stats* out) {
  if (!c || !out) return c ? fail(c, TKV_EINVAL, "tkv_get_stats: NULL") : TKV_EINVAL;
  tkv_status s = harvest_profile(c); if (s) return s;
  for (int t = 0; t < 4; ++t) c->st.tier_count[t] = c->ntier[t];
  c->st.host_rows_used = c->host_next;
  *out = c->st;
  return TKV_OK;
}

}  // extern "C"
