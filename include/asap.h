/*
 * asap.h -- C ABI of the MI355X (gfx950) visual-token pruning stage of ASAP
 * ("Attention-Shift-Aware Pruning", Sec. 4: salience-guided selection, Sec. 4.2:
 * salience-weighted consolidation).  Plain C: pointers, sizes, enums; no C++ or
 * framework types.  Every data pointer is a DEVICE pointer unless marked [host].
 *
 * One pruning stage = four calls on one stream, no host synchronisation between:
 *   asap_score      Eq. 2-5  -> raw mass s, salience s_hat, selection score r
 *   asap_select     top-k of r                                  (Fig. 3, stage 1)
 *   asap_merge      cosine routing + Eq. 6 + output sequence    (Sec. 4.2)
 *   asap_compact_kv K/V rows of the surviving positions         (KV-cache compatibility)
 *
 * Sequence layout of one image: P prefix tokens | V visual tokens | Tmax text slots
 * (text_len[b] <= Tmax of them valid), N = P + V + Tmax.  Visual-local index j is
 * sequence position P + j.  All index arrays are int32.
 *
 * Ownership: the caller owns every buffer including the workspace; the library
 * allocates nothing on the device, never synchronises the stream and keeps no
 * state between calls except the last error text of a context (and, once
 * asap_stage has been asked for two streams, that context's second stream and
 * three events, released by asap_destroy).
 * Errors: shapes, dtypes, pointers and workspace size are checked on the host
 * before anything is launched; a failed check launches nothing.  Contents of device
 * buffers (NaNs, text_len outside [1, Tmax]) are not checked.
 * Determinism: the same inputs give bit-identical outputs on every call.
 */
#ifndef ASAP_H
#define ASAP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct asap_ctx asap_ctx;   /* opaque: device id + last error text */

typedef enum {
  ASAP_OK = 0,
  ASAP_EINVAL = 1,        /* bad shape / pointer / alignment / parameter          */
  ASAP_EUNSUPPORTED = 2,  /* legal request this build has no kernel for           */
  ASAP_EWORKSPACE = 3,    /* workspace smaller than asap_workspace_bytes()        */
  ASAP_EHIP = 4           /* the HIP runtime refused a launch or a query          */
} asap_status;

typedef enum { ASAP_F32 = 0, ASAP_BF16 = 1 } asap_dtype;

/* How Eq. 4's discount enters the text->visual scores.
 * OFF:     no discount (plain attention-received top-k, the ablation's starting point).
 * KEYBIAS: ln(max(lambda_max * s_hat_j, eps)) is added to every text row's logit of key j,
 *          i.e. the unnormalised weight is lambda_j * exp(W_tj) (the exponent rule below Eq. 5). */
typedef enum { ASAP_MASK_OFF = 0, ASAP_MASK_KEYBIAS = 1 } asap_mask_mode;

/* ABSORB: every pruned token is routed to its most similar kept token.
 * PAPER: the consolidation of Sec. 4.2 as written -- redundancy is removed inside the kept set
 * (a kept token merges into a more salient, sufficiently similar kept token) and the vacated
 * slots are refilled with the pruned tokens of largest raw mass; see asap_merge.
 * PAPER needs k <= V / 2. */
typedef enum { ASAP_ROUTE_ABSORB = 0, ASAP_ROUTE_PAPER = 1 } asap_route;

/* Which text rows rank the visual tokens (Sec. 4.1 leaves it open).
 * ALL:  the mean over every valid text row (rows 0 .. text_len[b]-1 of q_txt).
 * LAST: the last valid text token's row alone (row text_len[b]-1), the criterion of plain
 *       attention-score pruning, the first rung of the ablation in Sec. 5.3. */
typedef enum { ASAP_ROWS_ALL = 0, ASAP_ROWS_LAST = 1 } asap_score_rows;

typedef struct {
  int32_t B;        /* images in the batch                                   >= 1 */
  int32_t H;        /* query heads                                                */
  int32_t Hkv;      /* key/value heads, H % Hkv == 0; head h reads kv head h*Hkv/H */
  int32_t d;        /* head dim, 64 or 128                                        */
  int32_t D;        /* hidden size, multiple of 64                                */
  int32_t P;        /* prefix tokens before the image, 0 .. 1048576               */
  int32_t V;        /* visual tokens, 1 .. 16384                                  */
  int32_t Tmax;     /* padded text length, 1 .. 128                               */
  int32_t k;        /* visual tokens kept, 1 .. V                                 */
  asap_dtype qk_dtype;   /* Q and K of the pruning layer                          */
  asap_dtype h_dtype;    /* hidden states in and out                              */
  asap_dtype kv_dtype;   /* K/V caches of the layers in front                     */
  float lambda_max;      /* Eq. 4, (0, 1]; 1.0 when the paper gives none          */
  float eps;             /* Eq. 3 and Eq. 4, > 0; the paper's 1e-6                */
  float sim_threshold;   /* t of Sec. 4.2: route only if cosine > t; -INFINITY = always */
  float merge_weight;    /* mu >= 0 on the source terms of Eq. 6; 1 = Eq. 6, 0 = no merging */
  asap_mask_mode mask_mode;
  asap_route route;
  asap_score_rows score_rows;
} asap_params;

/* Context for one device.  [host] pointers.  asap_create checks that `device` exists and
 * is a gfx950 part.  A context may be used from one thread at a time. */
asap_status asap_create(asap_ctx** out_ctx, int device);
void        asap_destroy(asap_ctx* ctx);
/* Text of the last error on this context ("" if none); valid until the next call on it. */
const char* asap_last_error(const asap_ctx* ctx);

/* Checks a parameter block on the host; msg (nullable, [host]) receives up to msg_len-1
 * characters naming the offending field. */
asap_status asap_check_params(const asap_params* p, char* msg, size_t msg_len);

/* Bytes of device scratch any of the four calls may need for these parameters (one size
 * serves all four).  0 if the parameters are invalid.  The workspace must be 256-byte
 * aligned; its contents are undefined before and after each call.  With f32 queries and keys it
 * includes 4 B H Tmax V bytes for the text rows' logits (Eq. 5), which are then formed once instead
 * of twice, unless that alone would exceed 1 GiB. */
size_t asap_workspace_bytes(const asap_params* p);

/*
 * asap_score -- Eq. 2, 3, 4, 5 and the selection score.
 *   s[b,j]     = 1/(H sqrt(d)) * sum_h sum_{i<V} q_vis[b,h,i,:] . k_vis[b,g(h),j,:]        (Eq. 2, mean over heads)
 *   s_hat[b,j] = (s - min_j s) / (max_j s - min_j s + eps)                                  (Eq. 3)
 *   lam[b,j]   = max(lambda_max * s_hat, eps)   (KEYBIAS)   or 1   (OFF)                    (Eq. 4)
 *   A[b,h,t,j] = lam_j exp(z_tj) / (sum_j' lam_j' exp(z_tj') + exp(lse_extra[b,h,t])),
 *                z_tj = q_txt[b,h,t,:] . k_vis[b,g(h),j,:] / sqrt(d)                        (Eq. 5, text rows)
 *   score[b,j] = 1/(H text_len[b]) * sum_h sum_{t<text_len[b]} A[b,h,t,j]
 *                (ASAP_ROWS_LAST: the one row t = text_len[b]-1, and 1/H in front)
 * q_vis [B,H,V,d], q_txt [B,H,Tmax,d], k_vis [B,Hkv,V,d] in qk_dtype; each *_stride[3] gives
 * the element strides of the three outer dims (last dim contiguous) so that the three may be
 * views into [B,heads,N,d] tensors.  Pointers 16-byte aligned, strides multiples of 8 elements.
 * text_len [B] int32.  lse_extra: NULL, or [B,H,Tmax] f32 = log-sum-exp of each text row's
 * logits over its NON-visual keys (then A is the full-row softmax of Eq. 5); NULL drops that term.
 * Outputs s_raw, s_hat, score: [B,V] f32, contiguous.  Sums are carried in fp64 up to the
 * final rounding of s_raw / s_hat, and per-row softmax terms in fp32.
 * Rows of q_txt at or past text_len[b] are padding: they are never used, whatever they hold.
 * When the rows that rank are few (ASAP_ROWS_LAST, or (H / Hkv) * Tmax <= 28 with bf16 keys), their
 * logits are taken in the sweep that computes s and kept in the workspace, and the keys are read
 * twice instead of three times.
 */
asap_status asap_score(asap_ctx* ctx, const asap_params* p,
                       const void* q_vis, const int64_t q_vis_stride[3],
                       const void* q_txt, const int64_t q_txt_stride[3],
                       const void* k_vis, const int64_t k_vis_stride[3],
                       const int32_t* text_len, const float* lse_extra,
                       float* s_raw, float* s_hat, float* score,
                       void* workspace, size_t workspace_bytes, void* stream /* hipStream_t */);

/*
 * asap_score_from_hidden -- asap_score with the raw mass of Eq. 2 taken from the hidden states instead
 * of from the visual queries (Sec. 3.1: a query is q_m = R_{Theta,m} W_q x_m, and Eq. 2 only needs the
 * sum of the visual queries, which is linear in the hidden states): the front end of the stage for a
 * caller that has not materialised the visual queries.  The rotation pairs coordinates (c, c + d/2) of
 * every head at angle pos * rope_theta^(-2c/d).
 *   hidden [B,N,D] h_dtype with element strides hidden_stride[2] (visual rows start at P);
 *   w_q [H*d, D] h_dtype, contiguous (row e = the weights of query coordinate e, i.e. q = W_q x);
 *   vis_positions: NULL (visual token i sits at position P + i) or [B,V] int32 position ids (a second
 *   stage keeps the original ids of its survivors);
 *   q_txt, k_vis, text_len, lse_extra, the outputs and every rule as for asap_score.
 * The workspace needs asap_front_end_workspace_bytes(p) bytes, 256-byte aligned.  The trigonometric
 * weights are taken in fp64 and rounded to f32; token sums run in fp32 over 64 tokens and in fp64 above.
 * The call reads the visual hidden states (B V D elements) where asap_score reads the visual queries
 * (B H V d elements) and does 2 d V D more multiply-adds per image: it is there for completeness of
 * the path, not for speed.
 */
size_t      asap_front_end_workspace_bytes(const asap_params* p);
asap_status asap_score_from_hidden(asap_ctx* ctx, const asap_params* p,
                                   const void* hidden, const int64_t hidden_stride[2],
                                   const void* w_q, double rope_theta, const int32_t* vis_positions,
                                   const void* q_txt, const int64_t q_txt_stride[3],
                                   const void* k_vis, const int64_t k_vis_stride[3],
                                   const int32_t* text_len, const float* lse_extra,
                                   float* s_raw, float* s_hat, float* score,
                                   void* workspace, size_t workspace_bytes, void* stream /* hipStream_t */);

/*
 * asap_score_static -- asap_score for callers that cannot allocate device memory and have no
 * workspace to hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Arguments, results and checks are those of asap_score without the workspace (with f32
 * keys asap_score keeps the logits of the text rows in its workspace and this call does so only
 * where the array can hold them; otherwise it forms them a second time, and the scores of the two
 * calls then differ by rounding, within the tolerance of either); the scratch is an array of ASAP_STATIC_SCRATCH_BYTES bytes that is part of the library's code object
 * (every GPU the library runs on holds its own copy until the process ends; asap_create looks up
 * its address on the context's device).  The call allocates and frees nothing.
 * ASAP_EWORKSPACE if the parameters need more scratch than the array holds (the message names both
 * sizes; asap_score with a caller workspace then serves): the array covers every benchmark
 * configuration, e.g. 16 images x 32 heads x 2304 visual tokens x 64 text rows takes 5.8 MB.
 * All calls on one GPU share that GPU's array and nothing in it has to survive between calls, but two
 * calls that overlap in time on one GPU (different streams, different contexts, different threads)
 * race on it: keep them ordered.
 */
#define ASAP_STATIC_SCRATCH_BYTES (16u << 20)
asap_status asap_score_static(asap_ctx* ctx, const asap_params* p,
                              const void* q_vis, const int64_t q_vis_stride[3],
                              const void* q_txt, const int64_t q_txt_stride[3],
                              const void* k_vis, const int64_t k_vis_stride[3],
                              const int32_t* text_len, const float* lse_extra,
                              float* s_raw, float* s_hat, float* score, void* stream /* hipStream_t */);

/*
 * asap_select -- the k largest score[b,:] per image, ties to the smaller index (Fig. 3, first
 * stage: only the k most salient visual tokens go on).  score [B,V] f32, finite and >= 0.
 * kept_idx [B,k] and pruned_idx [B,V-k]: visual-local indices, each ascending.
 */
asap_status asap_select(asap_ctx* ctx, const asap_params* p, const float* score,
                        int32_t* kept_idx, int32_t* pruned_idx,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * asap_merge -- Sec. 4.2 routing, Eq. 6, and the output sequence.  With ASAP_ROUTE_ABSORB:
 *   c(j,i)    = x_j . x_i / (max(|x_j|,1e-8) max(|x_i|,1e-8))   for pruned j, kept i (hidden states)
 *   assign[j] = slot (0..k-1, position in kept_idx) of the kept token with the largest c(j,.),
 *               ties to the smaller slot; -1 if that c <= sim_threshold.  best_sim[j] = that c.
 *   y_c       = (s_hat_i x_i + mu sum_{assign[j]=c} s_hat_j x_j) / wsum_c,
 *   wsum_c    = s_hat_i + mu sum s_hat_j;  a slot that absorbs no weight keeps x_i bit-exactly.  (Eq. 6)
 *   out_hidden[b] = prefix rows | y_0..y_{k-1} | text rows 0..text_len[b]-1   (Fig. 3: text and
 *               system prompt preserved); rows past new_len[b] = P + k + text_len[b] are not written.
 *   pos_out[b,n]  = original position id of output row n (n < new_len[b]), -1 beyond.
 * hidden [B,N,D] h_dtype with element strides hidden_stride[2] for (b, row); out_hidden
 * [B,P+k+Tmax,D] contiguous, h_dtype; must not overlap hidden.  s_hat [B,V] f32 from asap_score.
 * Dot products run on the matrix cores in the input precision (bf16 x bf16 or f32 x f32) with fp32
 * accumulation; Eq. 6 accumulates in fp32 and rounds once (nearest-even) to h_dtype.
 * assign [B,V-k] int32, best_sim [B,V-k] f32, wsum [B,k] f32, final_idx [B,k] int32 (= kept_idx here).
 * s_raw [B,V] f32 from asap_score is read only with ASAP_ROUTE_PAPER (NULL allowed otherwise).
 *
 * With ASAP_ROUTE_PAPER (Sec. 4.2 as written), for kept tokens i, j with cosine c(j,i) as above:
 *   j is a source iff some kept i has c(j,i) > sim_threshold and is stronger than j
 *     (s_hat_i > s_hat_j, ties to the smaller index); it goes to the most similar such i (ties to
 *     the smaller index) and chains are followed to their root, so each tree merges into one token
 *     that is not itself a source;
 *   the a vacated slots are refilled with the a pruned tokens of largest s_raw (ties to the
 *     smaller index), which stay unmerged;
 *   final_idx [B,k] = roots and refills, ascending; Eq. 6 over each root's tree; output sequence,
 *     pos_out, new_len as above with final_idx in the place of kept_idx.
 *   assign and best_sim then describe the kept tokens, laid out [B,k] at the start of the buffers:
 *     assign[b,a] = slot in final_idx of the root that absorbs kept_idx[b,a], -1 if it survives;
 *     best_sim[b,a] = cosine to its immediate destination (the best stronger token), -inf if none.
 */
asap_status asap_merge(asap_ctx* ctx, const asap_params* p,
                       const void* hidden, const int64_t hidden_stride[2],
                       const float* s_raw, const float* s_hat, const int32_t* text_len,
                       const int32_t* kept_idx, const int32_t* pruned_idx,
                       void* out_hidden, int32_t* pos_out, int32_t* new_len,
                       int32_t* assign, float* best_sim, float* wsum, int32_t* final_idx,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * asap_positions -- pos_out and new_len of the output sequence, from the kept set alone.
 * The stage keeps the survivors in their original order between the preserved prefix and text
 * (Fig. 3, Sec. 4.2), and with ASAP_ROUTE_ABSORB every kept token survives, so
 *   pos_out[b,n] = n (n < P);  P + kept_idx[b,n-P] (n < P+k);  P + V + (n-P-k) (n < new_len[b]);  -1 beyond,
 *   new_len[b]   = P + k + text_len[b]
 * are known as soon as asap_select has run.  A caller may therefore start asap_compact_kv (on
 * another stream) before or while asap_merge runs; asap_merge writes the same values into its own
 * pos_out / new_len.  kept_idx [B,k], text_len [B], pos_out [B,P+k+Tmax], new_len [B], int32, device.
 * ASAP_EUNSUPPORTED for any other route.
 */
asap_status asap_positions(asap_ctx* ctx, const asap_params* p, const int32_t* kept_idx,
                           const int32_t* text_len, int32_t* pos_out, int32_t* new_len, void* stream);

/*
 * asap_compact_kv -- drops the pruned tokens from the K/V caches of the n_layers layers in
 * front of the pruning layer: for every layer, K and V, image b and kv head g,
 *   dst[b,g,n,:] = src[b,g,pos_out[b,n],:]   for n < new_len[b]      (bit-exact copy)
 * Rows of kept tokens are copied unchanged (only the hidden state is merged).
 * k_src, v_src, k_dst, v_dst: [host] arrays of n_layers DEVICE pointers; src [B,Hkv,N,d],
 * dst [B,Hkv,P+k+Tmax,d], kv_dtype, contiguous, 16-byte aligned; dst must not overlap src.
 * pos_out [B,P+k+Tmax], new_len [B] from asap_merge or asap_positions.  1 <= n_layers <= 64.
 */
asap_status asap_compact_kv(asap_ctx* ctx, const asap_params* p, int32_t n_layers,
                            const void* const* k_src, const void* const* v_src,
                            void* const* k_dst, void* const* v_dst,
                            const int32_t* pos_out, const int32_t* new_len, void* stream);

/*
 * asap_compact_kv_from_kept -- asap_compact_kv without pos_out: the source rows are taken from the
 * list of surviving visual tokens and text_len, following the output order of the stage (Fig. 3:
 * prefix and text preserved around the kept tokens in their original order):
 *   dst[b,g,n,:]     = src[b,g,n,:]                      n < P
 *   dst[b,g,P+a,:]   = src[b,g,P+final_idx[b,a],:]       a < k
 *   dst[b,g,P+k+t,:] = src[b,g,P+V+t,:]                  t < text_len[b]
 * final_idx [B,k] int32 ascending = kept_idx of asap_select with ASAP_ROUTE_ABSORB, so the call can
 * be issued (on another stream) as soon as asap_select has run, without asap_positions in between;
 * final_idx of asap_merge with ASAP_ROUTE_PAPER.  Writes exactly what asap_compact_kv writes.
 * Buffers and limits as for asap_compact_kv.
 */
asap_status asap_compact_kv_from_kept(asap_ctx* ctx, const asap_params* p, int32_t n_layers,
                                      const void* const* k_src, const void* const* v_src,
                                      void* const* k_dst, void* const* v_dst,
                                      const int32_t* final_idx, const int32_t* text_len, void* stream);

/* Where asap_stage runs the K/V compaction: after the merge on the caller's stream, beside similarity
 * search and merge on a second stream, or on whichever of the two the sizes favour. */
typedef enum { ASAP_STREAMS_ONE = 0, ASAP_STREAMS_AUTO = 1, ASAP_STREAMS_TWO = 2 } asap_stream_mode;

/*
 * asap_stage -- the whole stage in one call: asap_score, asap_select, asap_merge and the K/V
 * compaction (asap_compact_kv_from_kept), with the arguments of those calls gathered in one struct
 * (same meaning, layout and checks; every check runs before the first launch).  n_layers = 0 skips
 * the compaction (the four K/V arrays may then be NULL).
 * two_streams (asap_stream_mode) and ASAP_ROUTE_ABSORB: the K/V rows depend on the kept set only,
 * so after the selection the compaction can be launched on a second stream of the context (default
 * priority, made on first use) ordered after `stream` by an event, next to the similarity and merge
 * kernels; `stream` waits for it at the end: work enqueued on `stream` after the call sees all
 * outputs.  The similarity kernel is bound on chip and the compaction by HBM, which is why the two
 * go well side by side.  ASAP_STREAMS_ONE never does this, ASAP_STREAMS_TWO always, and
 * ASAP_STREAMS_AUTO when the compaction moves at least 64 MiB (bytes read + written): below that
 * the two hand-overs between the streams cost more than they save.
 * The K/V rows that no selection can change (prefix, valid text; Fig. 3) do not wait for the
 * selection: when the caches are deep (the compaction moves more than four times the bytes of the
 * hidden states) the second stream starts on them at the beginning of the call, beside the score
 * kernels; else, for bf16 hidden states, B >= 12 and n_layers <= 16, further workgroups of the
 * launch that selects copy them.  The second stream then moves the rows of the kept tokens only;
 * the bytes written are the same in every case.
 * With ASAP_ROUTE_PAPER (final_idx exists only after the merge) everything runs on `stream` in
 * order.  Any other value of two_streams: ASAP_EINVAL.  One context must not run two stages at once.
 * The calls are capturable into a HIP graph (kernels, event record / wait; no memset, no sync).
 */
typedef struct asap_stage_io {
  /* asap_score */
  const void* q_vis;  int64_t q_vis_stride[3];
  const void* q_txt;  int64_t q_txt_stride[3];
  const void* k_vis;  int64_t k_vis_stride[3];
  const int32_t* text_len;
  const float* lse_extra;                      /* may be NULL */
  float* s_raw;  float* s_hat;  float* score;
  /* asap_select */
  int32_t* kept_idx;  int32_t* pruned_idx;
  /* asap_merge */
  const void* hidden;  int64_t hidden_stride[2];
  void* out_hidden;  int32_t* pos_out;  int32_t* new_len;
  int32_t* assign;  float* best_sim;  float* wsum;  int32_t* final_idx;
  /* K/V compaction: [host] arrays of n_layers device pointers, as for asap_compact_kv */
  int32_t n_layers;
  const void* const* k_src;  const void* const* v_src;
  void* const* k_dst;  void* const* v_dst;
  /* asap_workspace_bytes(p) bytes, 256-byte aligned */
  void* workspace;  size_t workspace_bytes;
} asap_stage_io;

asap_status asap_stage(asap_ctx* ctx, const asap_params* p, const asap_stage_io* io, int32_t two_streams,
                       void* stream);

/*
 * asap_compact_kv_paged -- asap_compact_kv for caches kept as pools of fixed-size pages with one
 * block table per sequence (the layout of paged serving engines; the paper fixes no cache layout, its
 * efficiency analysis only counts the K/V storage the pruned rows free).  A pool is
 * [n_pages, Hkv, page_size, d] in kv_dtype, contiguous, 16-byte aligned; token n of image b lives in
 * page table[b * table_stride + n / page_size] at slot n % page_size.  For every layer, K and V:
 *   dst_pool[dst_table[b, n / page_size], g, n % page_size, :] =
 *   src_pool[src_table[b, m / page_size], g, m % page_size, :],  m = pos_out[b,n],  n < new_len[b]
 * (bit-exact copy); no other slot of a destination pool is written.  Out of place: a destination
 * page must not be a source page of any sequence of the batch, but both tables may index one pool
 * (k_dst_pool[l] == k_src_pool[l] is allowed).  Tables are int32 device arrays shared by all
 * layers; src_table_stride >= ceil((P+V+Tmax) / page_size), dst_table_stride >=
 * ceil((P+k+Tmax) / page_size); page numbers are not checked against the pool sizes, which the
 * library does not know.  *_pool: [host] arrays of n_layers DEVICE pointers.  1 <= n_layers <= 64.
 */
asap_status asap_compact_kv_paged(asap_ctx* ctx, const asap_params* p, int32_t n_layers,
                                  const void* const* k_src_pool, const void* const* v_src_pool,
                                  void* const* k_dst_pool, void* const* v_dst_pool, int32_t page_size,
                                  const int32_t* src_table, int32_t src_table_stride,
                                  const int32_t* dst_table, int32_t dst_table_stride,
                                  const int32_t* pos_out, const int32_t* new_len, void* stream);

/*
 * asap_attention -- the attention forward of one decoder layer in front of the pruning layer under
 * the salience-guided bidirectional mask (Sec. 4.1, Eq. 4-5 applied to the whole sequence):
 *   out[b,h,i,:] = sum_j A_ij v[b,g(h),j,:],   A_i. = softmax_j( q[b,h,i,:] . k[b,g(h),j,:] / sqrt(d) + M_ij ),
 *   M_ij = 0                                         for j <= i                       (causal part, Eq. 1)
 *        = ln( max(lambda_max * s_hat[b,j-P], eps) ) for j > i, P <= i, j < P + V     (image span, Eq. 4)
 *        = -inf                                      otherwise;
 * with ASAP_MASK_OFF the second case is -inf too (plain causal attention).  N = P + V + Tmax rows,
 * all treated as valid.  q [B,H,N,d], k, v [B,Hkv,N,d] in qk_dtype with element strides of the
 * three outer dims (last dim contiguous; strides multiples of 8 elements), 16-byte aligned;
 * s_hat [B,V] f32 = the salience asap_score returns for this layer's q, k (NULL allowed with
 * ASAP_MASK_OFF); out [B,H,N,d] contiguous, qk_dtype.  Both contractions run on the matrix cores in
 * the input precision with fp32 accumulation; the probabilities are rounded to the input precision
 * before the second one.  The workspace (256-byte aligned) holds the per-key log discounts and,
 * except for bf16 with d = 128 (whose values are read in place), a transposed copy of v:
 * asap_attention_workspace_bytes(p) bytes.
 */
size_t      asap_attention_workspace_bytes(const asap_params* p);
asap_status asap_attention(asap_ctx* ctx, const asap_params* p,
                           const void* q, const int64_t q_stride[3],
                           const void* k, const int64_t k_stride[3],
                           const void* v, const int64_t v_stride[3],
                           const float* s_hat, void* out,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Theoretical FLOPs of the image tokens (Sec. 5, Eq. 7) for a pruning schedule of n_stages
 * stages, stage n running layers[n] decoder layers on tokens[n] image tokens, hidden size d and
 * FFN intermediate size m:
 *   flops = sum_n layers[n] * (4 v_n d^2 + 2 v_n^2 d + 3 v_n d m),   v_n = tokens[n]
 * and their ratio (Eq. 8) to the cost of all the layers at v0 tokens.  Host-side arithmetic in
 * double; layers, tokens [host], n_stages >= 1, every entry >= 0, d, m, v0 >= 1.
 */
asap_status asap_theoretical_flops(const int32_t* layers, const int32_t* tokens, int32_t n_stages,
                                   int32_t d, int32_t m, double* flops);
asap_status asap_flops_ratio(const int32_t* layers, const int32_t* tokens, int32_t n_stages,
                             int32_t v0, int32_t d, int32_t m, double* ratio);

/*
 * Kernel timing for benchmarks (not part of the method).  asap_timing_enable(ctx, n) with n > 0
 * creates a pool of n event pairs (n <= 8192); from then on each kernel the four calls launch
 * is bracketed by two HIP events recorded on the call's own stream, until the pool is used up
 * (later launches run untimed).  n <= 0 switches timing off and frees the pool.
 * asap_timing_collect waits for the recorded events, adds the elapsed times up per kernel name
 * and empties the pool for reuse: names [host] receives the kernel names, one per line;
 * total_ms[i] / launches[i] [host] the summed milliseconds and launch count of the i-th name.
 * Returns the number of distinct kernels (<= max_kernels, <= 64), or -1 on error.
 */
asap_status asap_timing_enable(asap_ctx* ctx, int32_t max_launches);
int32_t     asap_timing_collect(asap_ctx* ctx, char* names, size_t names_len, double* total_ms,
                                int32_t* launches, int32_t max_kernels);

#ifdef __cplusplus
}
#endif
#endif /* ASAP_H */
