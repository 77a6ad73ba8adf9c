// Host-side launch entry points of the kernel files (internal; the public ABI is asap.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <type_traits>

#include "asap.h"

namespace asap {

// Carve-up of the caller's workspace for the score path.  All offsets 256-byte aligned.
struct ScoreWorkspace {
  int q_rows;        // visual query rows summed per k_qsum block
  int q_chunks;      // ceil(V / q_rows)
  int attn_splits;   // key-range splits of the text-row sweeps
  int t_eff;         // text rows that rank the tokens: Tmax, or 1 with ASAP_ROWS_LAST
  int ride;          // 1: those rows ride in the mass sweep, which leaves their logits (no text-row sweeps)
  int row_pairs;     // pairs of 32-row blocks of text queries, each with sweep workgroups of its own
  int head_splits;   // kv-head groups of the mass sweep with workgroups of their own (small batches)
  int store_logits;  // 1: the first text-row sweep leaves its logits and the column sums read those
  size_t off_qpart;  // double [B,H,q_chunks,d]  partial sums of visual queries
  size_t off_qbar;   // double [B,Hkv,d]         summed visual queries per kv head
  size_t off_qsplit; // bf16   [B,Hkv,4,d]       the same, split into four bf16 pieces per component
  size_t off_s64;    // double [B,V]             raw attention mass before rounding
  size_t off_mm;     // uint64 [B,2]             order-preserving keys of min, max of s per image
  size_t off_pstat;  // float  [B,H,splits,2,NR] per-split (max, sum) of every text row, NR = 64 row_pairs
  size_t off_upart;  // float  [B,H,row_pairs,V] column sums of normalised weights per head and row pair
  size_t off_spart;  // double [head_splits,B,V] partial masses (head_splits > 1)
  size_t off_zlog;   // float  [B,H,t_eff,V]     raw logits of the ranking rows (ride, store_logits)
  size_t total;
};
// budget: the bytes the caller can give; optional parts of the workspace (the stored logits) are
// planned only if the whole then fits.
constexpr size_t STORED_LOGITS_MAX_BYTES = size_t(1) << 30;
ScoreWorkspace score_workspace(const asap_params& p, size_t budget = ~size_t(0));

struct Strides3 { int64_t b, h, r; };

// Optional per-kernel timing: when a Timer is passed, every kernel launch is bracketed by two HIP
// events recorded on the launch stream.  Events come from a fixed pool; when it is used up further
// launches go untimed.
struct Timer {
  static constexpr int kMaxRecords = 8192;
  struct Record { const char* name; hipEvent_t start, stop; };
  Record rec[kMaxRecords];
  int n_created = 0;
  int n_used = 0;
  Record* begin(const char* name, hipStream_t st) {
    if (n_used >= n_created) return nullptr;
    Record* r = &rec[n_used++];
    r->name = name;
    (void)hipEventRecord(r->start, st);
    return r;
  }
  static void end(Record* r, hipStream_t st) {
    if (r) (void)hipEventRecord(r->stop, st);
  }
};

// Launches `kern` and, if `tm` is set, times it under `name`.
#define ASAP_LAUNCH(tm, name, kern, grid, block, lds, st, ...)                  \
  do {                                                                          \
    ::asap::Timer::Record* asap_rec_ = (tm) ? (tm)->begin(name, st) : nullptr;  \
    hipLaunchKernelGGL(kern, grid, block, lds, st, __VA_ARGS__);                \
    ::asap::Timer::end(asap_rec_, st);                                          \
  } while (0)

// Eq. 2 from hidden states (asap_front.hip): the summed visual queries are computed from the hidden
// states, W_q [H d, D] (h_dtype) and the rotary angles instead of from the visual queries.
struct FrontArgs {
  const void* hidden; int64_t hsb, hsr;   // [B,N,D] h_dtype, element strides
  const void* wq;                         // [H*d, D] h_dtype, contiguous
  double rope_theta;
  const int32_t* vis_positions;           // [B,V] position ids of the visual tokens, or null: P + i
  char* ws;                               // front_workspace_bytes(p)
};
size_t front_workspace_bytes(const asap_params& p);
hipError_t launch_front_end(const asap_params& p, const void* hidden, int64_t hsb, int64_t hsr, const void* wq,
                            double rope_theta, const int32_t* vis_positions, double* qpart, char* ws, hipStream_t st,
                            Timer* tm);

// K and V of up to 16 cached layers, K then V of each layer.
constexpr int KV_LAYERS_PER_LAUNCH = 16;
struct KvPointers {
  const char* src[2 * KV_LAYERS_PER_LAUNCH];
  char* dst[2 * KV_LAYERS_PER_LAUNCH];
};
// The K/V rows that survive whatever the selection keeps (Fig. 3: the prefix and the valid text rows),
// for the launch that moves them while the selection runs.
struct KvFixedRows {
  KvPointers ptrs;
  int n_bufs;                 // 2 * layers
  int Hkv, N, Nout, row_bytes, P, V, k, Tmax;
};
void fill_kv_pointers(KvPointers* ptrs, int n_layers, const void* const* k_src, const void* const* v_src,
                      void* const* k_dst, void* const* v_dst);

// The selection rides in the launch that finishes the score when the batch gives that launch (one
// workgroup per image) enough workgroups to fetch the per-head sums at a reasonable rate; measured
// on batches of 4 and 8 it lost to the two separate launches.
inline bool score_fuses_selection(const asap_params& p) { return p.B >= 12; }

// kept != nullptr: the top-k selection runs in the launch that finishes the score (the stage as one
// call), writing kept [B,k] and pruned [B,V-k] exactly as launch_select would.  fixed != nullptr (only
// with kept and score_fuses_selection(p)): further workgroups of that launch copy the K/V rows of the
// prefix and of the valid text, which depend on no result, while the memory system is otherwise idle.
// ws_budget: the budget score_workspace planned ws with (~0 for workspaces sized by asap_workspace_bytes).
hipError_t launch_score(const asap_params& p, const void* q_vis, Strides3 qv, const void* q_txt, Strides3 qt,
                        const void* k_vis, Strides3 kv, const int32_t* text_len, const float* lse_extra,
                        float* s_raw, float* s_hat, float* score, int32_t* kept, int32_t* pruned,
                        const FrontArgs* fe, const KvFixedRows* fixed, char* ws, size_t ws_budget,
                        hipStream_t st, Timer* tm);

hipError_t launch_select(const asap_params& p, const float* score, int32_t* kept, int32_t* pruned,
                         hipStream_t st, Timer* tm);

hipError_t launch_merge(const asap_params& p, const void* hidden, int64_t hsb, int64_t hsr, const float* s_raw,
                        const float* s_hat, const int32_t* text_len, const int32_t* kept, const int32_t* pruned,
                        void* out_hidden, int32_t* pos_out, int32_t* new_len, int32_t* assign, float* best_sim,
                        float* wsum, int32_t* final_idx, char* ws, hipStream_t st, Timer* tm);

// Cosine routing (asap_sim.hip): for each of the M source tokens srcs[b,:] the most similar kept
// token (slot in kept, -1 if the similarity does not exceed the threshold) and that similarity.
// anchored: the routing inside the kept set of Sec. 4.2 (srcs = kept, M = k): only destinations
// stronger than the source count, by s_hat [B,V] and then by index.  ws: sim_workspace_bytes(p).
size_t sim_workspace_bytes(const asap_params& p);
hipError_t launch_similarity(const asap_params& p, const void* hidden, int64_t hsb, int64_t hsr,
                             const int32_t* kept, const int32_t* srcs, int M, bool anchored, const float* s_hat,
                             int32_t* assign, float* best_sim, char* ws, hipStream_t st, Timer* tm);

// Second half of the paper's routing (asap_paper.hip): chains of destinations followed to their
// roots, the vacated slots refilled with the pruned tokens of largest raw mass, the final kept list
// and, per kept slot, the slot of the final token that absorbs it (-1: it survives).
size_t paper_workspace_bytes(const asap_params& p);
hipError_t launch_paper_plan(const asap_params& p, const int32_t* dest, const int32_t* kept, const float* s_raw,
                             int32_t* final_idx, int32_t* assign, hipStream_t st, Timer* tm);

hipError_t launch_positions(const asap_params& p, const int32_t* kept, const int32_t* text_len, int32_t* pos_out,
                            int32_t* new_len, hipStream_t st, Timer* tm);

// KV_BY_POS: idx = pos_out, len = new_len; KV_FROM_KEPT: idx = kept list, len = text_len, all output
// rows; KV_KEPT_ONLY: as KV_FROM_KEPT but only the rows of the kept tokens; KV_FIXED_ONLY: the other
// rows (prefix, valid text), which need no index list.  The last two together move what KV_FROM_KEPT
// moves.
enum { KV_BY_POS = 0, KV_FROM_KEPT = 1, KV_KEPT_ONLY = 2, KV_FIXED_ONLY = 3 };
hipError_t launch_compact_kv(const asap_params& p, int mode, int n_layers, const void* const* k_src,
                             const void* const* v_src, void* const* k_dst, void* const* v_dst,
                             const int32_t* idx, const int32_t* len, hipStream_t st, Timer* tm);
hipError_t launch_compact_kv_paged(const asap_params& p, int n_layers, const void* const* k_src,
                                   const void* const* v_src, void* const* k_dst, void* const* v_dst, int page_size,
                                   const int32_t* src_table, int src_stride, const int32_t* dst_table,
                                   int dst_stride, const int32_t* pos_out, const int32_t* new_len, hipStream_t st,
                                   Timer* tm);

// attention forward under the Eq. 4-5 mask (asap_attention.hip); ws needs attention_workspace_bytes(p)
size_t attention_workspace_bytes(const asap_params& p);
hipError_t launch_attention(const asap_params& p, const void* q, Strides3 sq, const void* k, Strides3 sk,
                            const void* v, Strides3 sv, const float* s_hat, void* out, char* ws, hipStream_t st,
                            Timer* tm);

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

}  // namespace asap
