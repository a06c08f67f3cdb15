// Internal declarations shared by the host runtime and the gfx950 kernels of libtkv.
// Nothing here is part of the public ABI (see include/tkv.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tkv {

// ---- per-sequence counters kept on the device: cnt[b * CNT_N + k] -------------------------------
enum Cnt : int {
  C_NF = 0,      // entries of the full-precision list F = T0 u T1, ascending position
  C_NQ,          // entries of the compressed list Q = T2, ascending position
  C_N0, C_N1, C_N2, C_N3,   // positions per tier
  C_FREE0, C_FREE1, C_FREE2, // free slots on the stacks of the HBM pool, the staging buffer, the T2 pool
  C_PEND,        // HBM slots of rows that went T0->T1 at the last migrate; released at the next one
  // plan counts (written by plan_count, read by the host and by plan_commit)
  C_M01, C_M02, C_M03, C_M10, C_M12, C_M13, C_M20, C_M21, C_M23,
  C_BAD,         // positions that would leave T3 (invalid plan)
  C_LEN,         // positions assigned so far
  C_P0, C_P1, C_P2, C_P3,   // planned positions per tier (plan_count)
  C_M01R,        // of the T0->T1 moves, rows whose copy in the pinned store is still valid (no transfer: copied inside HBM)
  C_MCOPY,       // rows copied inside HBM: T1->T0 plus the T0->T1 moves counted in C_M01R
  C_NS,          // streamed T1: entries of the T1 list (list F then holds T0 alone)
  CNT_N = 29
};

constexpr int TOK_PER_BLOCK = 64;    // list entries per attention tile (one per lane of a wave)
constexpr int PLAN_THREADS = 1024;
constexpr int MAX_G = 8;
constexpr int ATTN_ARG_SEQS = 64;    // list lengths travel as kernel arguments up to this batch size

// Device view of one cache, passed by value to the tier-management kernels.
struct DevView {
  int L, B, Hq, Hkv, G, D;
  int Nmax;                 // max_tokens
  int cap0, cap1, cap2;     // slots per (layer, seq, kv head): HBM pool, staging buffer, compressed pool
  int capF;                 // cap0 + cap1: one slot space, staging slots are cap0 .. capF-1
  int es;                   // bytes per K/V element
  int kt;                   // 0 binary32, 1 bfloat16, 2 binary16
  int t2fmt;                // 0 int8 row, 1 int4 g32
  int cb, sb;               // bytes of codes / of scales per T2 row
  int n_prompt, k_sink, k_window;
  char* fpK; char* fpV;     // [L][B][Hkv][capF][D*es]
  char* c2K; char* c2V;     // [L][B][Hkv][cap2][cb]
  char* s2K; char* s2V;     // [L][B][Hkv][cap2][sb]
  uint8_t* tier;            // [B][Nmax] current
  uint8_t* tier_new;        // [B][Nmax] pending
  int* loc;                 // [B][Nmax] slot in the pool of the position's tier (T0/T1: unified F slot; T2: T2 slot; T3: -1)
  int* hloc;                // [B][Nmax] row in the pinned host store that holds the position's current bits (every T1 row,
                            // and T0 rows that came up from T1), else -1
  float* score;             // [B][Nmax]
  int* f_pos; int* f_loc;   // [B][Nmax] list F: position, slot
  int* f_loc_old;           // [B][Nmax] list F with the pre-offload slot of rows whose staged copy is still in flight
  int* q_pos; int* q_loc;   // [B][Nmax] list Q
  int* idx;                 // [4][B][Nmax] per-tier ascending position lists
  int* cnt;                 // [B][CNT_N]
  int* free0; int* free1; int* free2;  // [B][cap] stacks of free slots (free0/free1 hold unified F slots)
  int* pend;                // [B][Nmax]
  int* rel0; int* rel1; int* rel2;     // [B][Nmax] scratch: slots released by the plan being committed
  // move lists written by plan_commit (per sequence, [B][Nmax] each, counts in cnt)
  int* mv10_src; int* mv10_dst;    // copies inside the F slot space: staging slot -> HBM slot, and HBM slot -> staging slot for
                                   // rows that return to T1 with a valid host copy
  int* mvq_src; int* mvq_dst;      // F slot -> T2 slot (encode)
  int* mvd_src; int* mvd_dst;      // T2 slot -> HBM slot (decode)
  // rows going to the host store at this migrate, global order = host row order
  int* g_seq; int* g_src; int* g_dst;   // [host_rows_per_event]: sequence, HBM slot to read, staging slot to fill
  const int* host_base;     // [B] first host row of the sequence's rows at this migrate
  int event_base;           // first host row of this migrate
  // Streamed T1: the staging slots cap0 .. capF-1 are not backed per layer; one frame [B][Hkv][cap1][D*es] (K and V)
  // is refilled from the pinned store for the layer that is attended next.
  int streamed;             // != 0: streamed T1
  int capP;                 // rows per (layer, seq, kv head) of the pool fpK / fpV: capF, or cap0 when streamed
  char* frK; char* frV;     // the frame the row movers read staging slots from (set per launch)
  int* s_pos; int* s_loc;   // [B][Nmax] streamed: list of the T1 rows (position, frame slot = staging slot - cap0); list F
                            // then holds T0 alone
  int* h_seq; int* h_dst;   // [host_rows] streamed: for every row of the pinned store its sequence and the staging slot of
                            // the T1 position it belongs to (-1: the row's position is not in T1 any more)
  int* h_clr;               // [B][Nmax] scratch: host rows of the positions that leave T1 in the plan being committed
  float* vnorm;             // [L][B][Hkv][Nmax] value-aware scorer: Euclidean norm of every appended value row, by position
                            // (NULL with the attention-only scorer)
  float* red;               // [L][B][Hkv][Nmax] redundancy-penalised scorers: clamped cosine of every appended key row with
                            // the key row appended before it, by position (else NULL)
  char* last_k;             // [L][B][Hkv][D] the key row appended last, in the KV type (with red)
};

struct AttnArgs {
  const char* fpK; const char* fpV;   // layer bases
  const char* c2K; const char* c2V; const char* s2K; const char* s2V;
  const void* q; void* out;
  const int* f_loc; const int* f_pos; const int* q_loc; const int* q_pos;
  const int* cnt;
  float* score;
  float* xs;        // [B][Hkv][G][xs_stride] scaled logits by list index (F tiles, then Q tiles)
  float* part_ml;   // [B][Hkv][S][2][G]  (m, l) of each split (= workgroup)
  float* part_o;    // [B][Hkv][S][G][D]
  int S;            // workgroups per (sequence, kv head) of this launch
  int S_total, s0;  // splits the finishing kernel merges, and the first one this launch writes (streamed T1: a second
                    // launch serves the T1 rows from the staging frame and writes the splits after the first launch's)
  int second;       // != 0: that second launch; its list lengths are nS, its logits follow the first launch's tiles
  const int* s_pos; // [B][Nmax] positions of the T1 list (streamed T1), for the finishing kernel
  const float* vnorm; // [B][Hkv][Nmax] this layer's value-row norms (value-aware scorer), else NULL
  const float* red;   // [B][Hkv][Nmax] this layer's key redundancies (redundancy-penalised scorers), else NULL
  float red_w;        // weight of the redundancy penalty
  int n_tiles;      // max over the sequences of F tiles + Q tiles (+ T1 tiles)
  int q_bs, o_bs;   // query heads between consecutive sequences in q and in out: Hq, or n_q * Hq for the tokens of a chunk
  int trim;         // entries at the end of list F this call leaves out (the chunk's later tokens); nF[] has them
                    // taken off already, the device counter has not
  int n_q, cq;      // query tokens per sequence served by this launch: n_q groups along grid z (grid z = B * n_q) of cq
                    // tokens each (columns of one workgroup; 16-bit rows only, cq * G <= 32).  Token jt = jz * cq + jc of
                    // a sequence is jt * Hq heads further on in q and out, leaves n_q * cq - 1 - jt more entries of
                    // list F out (it is that many positions older), and has logits and split partials of its own
                    // (index b * n_q * cq + jt)
  int B, Hq, Hkv, Nmax, capF, cap2, xs_stride, cb, sb, t2fmt, out_kind, q_es;   // out_kind: 0 binary32, 1 bfloat16, 2 binary16
  float softmax_scale, score_scale;
  int nF[ATTN_ARG_SEQS], nQ[ATTN_ARG_SEQS];   // list lengths per sequence (host mirror), used when B <= ATTN_ARG_SEQS
  int nWq[ATTN_ARG_SEQS];                     // waves of each (sequence, kv head) pair that serve the Q list (same condition)
  // (streamed T1: the second launch and the finishing kernel take the T1 list's length and the first launch's tile
  // counts from the device counters; the argument block stays small, it is read over the host link in some set-ups)
};

// launchers (defined in the .hip files)
// kt: type of K, V and q (0 binary32, 1 bfloat16, 2 binary16)
hipError_t launch_attn_tiered(const AttnArgs& a, int D, int G, int kt, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1);
hipError_t launch_attn_finish(const AttnArgs& a, int D, int G, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1);
hipError_t launch_attn_finish_chunk(const AttnArgs& a, int D, int G, hipStream_t st);
int attn_cols_per_launch(int elem_bytes, int G);   // query tokens one workgroup can take as columns
hipError_t launch_probe_read(const void* src, size_t bytes, int workgroups, uint32_t* sink, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1);
int attn_waves_per_group(int D, int elem_bytes, int G, int cq = 1);   // waves per attention workgroup (one workgroup per compute unit)
int attn_q_waves(int n_waves, int n_f_tiles, int n_q_tiles);   // how many of a pair's waves serve the Q list
hipError_t launch_append(const DevView& v, int layer, const void* k, const void* v_, int pos0, int n_new,
                         bool assign, hipStream_t st);
hipError_t launch_append_step(const DevView& v, const void* k, const void* v_, int pos, hipStream_t st);
hipError_t launch_classify(const DevView& v, int n, const uint32_t* ppm, hipStream_t st);
hipError_t launch_plan_count(const DevView& v, int n, hipStream_t st);
hipError_t launch_plan_commit(const DevView& v, int n, hipStream_t st);
hipError_t launch_moves(const DevView& v, int max10, int maxq, int maxd, hipStream_t st);
// streamed T1: the two movers that may read staging slots, for one layer whose rows are in the frame v.frK / v.frV
hipError_t launch_moves_layer(const DevView& v, int layer, int max10, int maxq, hipStream_t st);
hipError_t launch_decode_moves(const DevView& v, int maxd, hipStream_t st);
hipError_t launch_clear_host_rows(const DevView& v, int max_leaving, hipStream_t st);
hipError_t launch_scatter_frame(const DevView& v, int r0, int nrows, const char* bounce, hipStream_t st);
hipError_t launch_rehome(const DevView& v, int n, hipStream_t st);
// streamed T1: new packed numbering of the T1 rows of the plan just committed (into g2_seq / g2_src / hloc2), and its adoption
hipError_t launch_repack_number(const DevView& v, int n, const int* base2, int* g2_seq, int* g2_src, int* hloc2, hipStream_t st);
hipError_t launch_repack_apply(const DevView& v, int n, const int* hloc2, hipStream_t st);
hipError_t launch_rebuild_htable(const DevView& v, int n, int rows, hipStream_t st);
hipError_t launch_gather(const DevView& v, int layer, int r0, int nrows, char* bounce, hipStream_t st);
hipError_t launch_scatter(const DevView& v, int layer, int r0, int nrows, const char* bounce, hipStream_t st);
hipError_t launch_init_state(const DevView& v, hipStream_t st);

}  // namespace tkv
