// asap_merge: the salience-weighted convex merge of Eq. 6 and the output sequence
// [prefix | merged kept | text], after the cosine routing of asap_sim.hip (and, for the paper's
// routing inside the kept set, the plan of asap_paper.hip).
//
//   k_merge<T>    one workgroup per output row: copies prefix / text rows, and for a final
//                 slot gathers its sources in ascending order and applies Eq. 6.  The sources are
//                 M candidate tokens with assign[] = the slot that absorbs each (or -1): the
//                 pruned tokens with ABSORB routing, the kept tokens with the paper's.
#include "asap_device.hpp"
#include "asap_launch.hpp"

namespace asap {

// ------------------------------------------------------------------------------------------
// k_merge: grid (P + k + Tmax, B), 256 threads.
// ------------------------------------------------------------------------------------------
constexpr int MERGE_SEG = 2048;   // entries of assign[] scanned per round

template <typename T, int CPT>    // CPT = 16-byte chunks of a row per thread (row = D elements)
__global__ __launch_bounds__(256) void k_merge(const T* __restrict__ hidden, int64_t sb, int64_t sr, int D,
                                                int P, int V, int k, int M, int Tmax, float mu,
                                                const float* __restrict__ s_hat, const int32_t* __restrict__ text_len,
                                                const int32_t* kept /* may be final_idx */,
                                                const int32_t* __restrict__ pruned,
                                                const int32_t* __restrict__ assign, T* __restrict__ out,
                                                int32_t* __restrict__ pos_out, int32_t* __restrict__ new_len,
                                                float* __restrict__ wsum, int32_t* final_idx) {
  constexpr int E = elem<T>::per16;
  __shared__ int list[MERGE_SEG];
  __shared__ int wave_cnt[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nrow = blockIdx.x, b = blockIdx.y;
  const int Nout = P + k + Tmax;
  const int len = text_len[b];
  const int nchunks = D / E;
  const char* hb = reinterpret_cast<const char*>(hidden + b * sb);
  const int64_t rowb = sr * (int64_t)sizeof(T);
  char* orow = reinterpret_cast<char*>(out + ((int64_t)b * Nout + nrow) * D);
  if (nrow == 0 && tid == 0) new_len[b] = P + k + len;

  if (nrow < P || nrow >= P + k) {                       // prefix or text row: plain copy
    int src;
    if (nrow < P) src = nrow;
    else {
      int t = nrow - P - k;
      src = (t < len) ? P + V + t : -1;
    }
    if (tid == 0) pos_out[(int64_t)b * Nout + nrow] = src;
    if (src < 0) return;
    const char* s = hb + (int64_t)src * rowb;
    for (int c = tid; c < nchunks; c += 256) stg16_stream(orow + c * 16, ldg16_stream(s + c * 16));
    return;
  }

  const int slot = nrow - P;
  const int i_tok = kept[(int64_t)b * k + slot];
  const float* sh = s_hat + (int64_t)b * V;
  const float w_i = sh[i_tok];
  const char* xrow = hb + (int64_t)(P + i_tok) * rowb;
  float acc[CPT][E];
#pragma unroll
  for (int q = 0; q < CPT; ++q) {
    int c = tid + q * 256;
    if (c < nchunks) {
      float f[E];
      unpack16<T>(ldg16_stream(xrow + c * 16), f);
#pragma unroll
      for (int e = 0; e < E; ++e) acc[q][e] = w_i * f[e];
    }
  }
  float den = w_i, absorbed = 0.0f;
  const int32_t* asg = assign + (int64_t)b * M;
  const int32_t* pr = pruned + (int64_t)b * M;
  for (int seg = 0; seg < M; seg += MERGE_SEG) {
    // ordered compaction of the sources of this slot among entries [seg, seg + MERGE_SEG)
    constexpr int PER = MERGE_SEG / 256;
    int mine[PER];
    int cnt = 0;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      int a = seg + tid * PER + e;
      mine[e] = -1;
      if (a < M && asg[a] == slot) { mine[e] = pr[a]; ++cnt; }
    }
    int incl = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      int y = __shfl_up(incl, off);
      if (lane >= off) incl += y;
    }
    __syncthreads();
    if (lane == 63) wave_cnt[wave] = incl;
    __syncthreads();
    int base = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      if (w < wave) base += wave_cnt[w];
      total += wave_cnt[w];
    }
    int pos = base + incl - cnt;
#pragma unroll
    for (int e = 0; e < PER; ++e)
      if (mine[e] >= 0) list[pos++] = mine[e];
    __syncthreads();
    for (int s0 = 0; s0 < total; s0 += 4) {
      uint4 ch[4][CPT];
      float w[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        int j = list[min(s0 + u, total - 1)];
        w[u] = (s0 + u < total) ? mu * sh[j] : 0.0f;
        const char* srow = hb + (int64_t)(P + j) * rowb;
#pragma unroll
        for (int q = 0; q < CPT; ++q) {
          int c = tid + q * 256;
          if (c < nchunks) ch[u][q] = ldg16_stream(srow + c * 16);
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (s0 + u < total) {
          den += w[u];
          absorbed += w[u];
#pragma unroll
          for (int q = 0; q < CPT; ++q) {
            int c = tid + q * 256;
            if (c < nchunks) {
              float f[E];
              unpack16<T>(ch[u][q], f);
#pragma unroll
              for (int e = 0; e < E; ++e) acc[q][e] = fmaf(w[u], f[e], acc[q][e]);
            }
          }
        }
      }
    }
  }
  if (tid == 0) {
    wsum[(int64_t)b * k + slot] = den;
    final_idx[(int64_t)b * k + slot] = i_tok;
    pos_out[(int64_t)b * Nout + nrow] = P + i_tok;
  }
  if (absorbed > 0.0f) {
    const float inv = 1.0f / den;
#pragma unroll
    for (int q = 0; q < CPT; ++q) {
      int c = tid + q * 256;
      if (c < nchunks) {
        float f[E];
#pragma unroll
        for (int e = 0; e < E; ++e) f[e] = acc[q][e] * inv;
        stg16_stream(orow + c * 16, pack16<T>(f));
      }
    }
  } else {                                               // nothing absorbed: Eq. 6 is the identity
    for (int c = tid; c < nchunks; c += 256) stg16_stream(orow + c * 16, ldg16_stream(xrow + c * 16));
  }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
template <typename T>
static hipError_t merge_typed(const asap_params& p, const void* hidden, int64_t hsb, int64_t hsr,
                              const float* s_hat, const int32_t* text_len, const int32_t* kept,
                              const int32_t* cand, int M, void* out_hidden, int32_t* pos_out, int32_t* new_len,
                              int32_t* assign, float* wsum, int32_t* final_idx, hipStream_t st, Timer* tm) {
  const T* h = static_cast<const T*>(hidden);
  constexpr int E = elem<T>::per16;
  const int nchunks = p.D / E;
  const int cpt = (nchunks + 255) / 256;
  dim3 grid(p.P + p.k + p.Tmax, p.B);
#define ASAP_MERGE(CPT)                                                                                    \
  ASAP_LAUNCH(tm, "k_merge", (k_merge<T, CPT>), grid, dim3(256), 0, st, h, hsb, hsr, p.D, p.P, p.V, p.k,   \
              M, p.Tmax, p.merge_weight, s_hat, text_len, kept, cand, assign, static_cast<T*>(out_hidden), \
              pos_out, new_len, wsum, final_idx)
  if (cpt <= 1) ASAP_MERGE(1);
  else if (cpt <= 2) ASAP_MERGE(2);
  else if (cpt <= 4) ASAP_MERGE(4);
  else if (cpt <= 8) ASAP_MERGE(8);
  else return hipErrorInvalidValue;
#undef ASAP_MERGE
  return hipGetLastError();
}

hipError_t launch_merge(const asap_params& p, const void* hidden, int64_t hsb, int64_t hsr, const float* s_raw,
                        const float* s_hat, const int32_t* text_len, const int32_t* kept, const int32_t* pruned,
                        void* out_hidden, int32_t* pos_out, int32_t* new_len, int32_t* assign, float* best_sim,
                        float* wsum, int32_t* final_idx, char* ws, hipStream_t st, Timer* tm) {
  const bool bf = p.h_dtype == ASAP_BF16;
  if (p.route == ASAP_ROUTE_PAPER) {
    // kept x kept search (destinations into the workspace) -> roots, refills, final list -> merge
    // with the kept tokens as candidates and the final list in the place of the kept list
    int32_t* dest = reinterpret_cast<int32_t*>(ws);
    hipError_t e = launch_similarity(p, hidden, hsb, hsr, kept, kept, p.k, true, s_hat, dest, best_sim,
                                     ws + paper_workspace_bytes(p), st, tm);
    if (e != hipSuccess) return e;
    e = launch_paper_plan(p, dest, kept, s_raw, final_idx, assign, st, tm);
    if (e != hipSuccess) return e;
    return bf ? merge_typed<bf16_t>(p, hidden, hsb, hsr, s_hat, text_len, final_idx, kept, p.k, out_hidden, pos_out,
                                    new_len, assign, wsum, final_idx, st, tm)
              : merge_typed<float>(p, hidden, hsb, hsr, s_hat, text_len, final_idx, kept, p.k, out_hidden, pos_out,
                                   new_len, assign, wsum, final_idx, st, tm);
  }
  const int M = p.V - p.k;
  if (M > 0) {
    hipError_t e = launch_similarity(p, hidden, hsb, hsr, kept, pruned, M, false, s_hat, assign, best_sim, ws, st, tm);
    if (e != hipSuccess) return e;
  }
  return bf ? merge_typed<bf16_t>(p, hidden, hsb, hsr, s_hat, text_len, kept, pruned, M, out_hidden, pos_out, new_len,
                                  assign, wsum, final_idx, st, tm)
            : merge_typed<float>(p, hidden, hsb, hsr, s_hat, text_len, kept, pruned, M, out_hidden, pos_out, new_len,
                                 assign, wsum, final_idx, st, tm);
}

}  // namespace asap
