// asap_merge: cosine routing of pruned tokens to kept tokens (Sec. 4.2), the salience-weighted
// convex merge of Eq. 6, and the output sequence [prefix | merged kept | text].
//
//   k_sim<T, NT>  per image: (pruned rows) x (kept rows)^T over the hidden dimension on the
//                 matrix cores, squared norms gathered on the way, fused row arg-max.
//   k_merge<T>    one workgroup per output row: copies prefix / text rows, and for a kept
//                 slot gathers its sources in ascending order and applies Eq. 6.
#include "asap_device.hpp"
#include "asap_launch.hpp"

namespace asap {

// ------------------------------------------------------------------------------------------
// k_sim.  Workgroup tile: BM = 128 source rows x BN = 64*NT destination rows, 256 threads =
// 2 x 2 waves, each wave 64 x 32*NT (2 x NT MFMA tiles of 32 x 32).  The hidden dimension is
// walked in steps of 128 bytes per row; a step's (BM + BN) x 128 B panel is staged through
// LDS (rows padded to 144 B), double buffered, one barrier per step.  Thread t moves the
// 16-byte piece t % 8 of rows t / 8 + 32 i and accumulates those rows' sums of squares.
// grid (ceil(M / 128), B).
// ------------------------------------------------------------------------------------------
constexpr int SIM_BM = 128;
constexpr int SIM_LDSROW = 144;

template <typename T, int NT>
__global__ __launch_bounds__(256) void k_sim(const T* __restrict__ xv, int64_t sb, int64_t sr, int D,
                                              const int32_t* __restrict__ pruned, const int32_t* __restrict__ kept,
                                              int M, int k, float threshold, int32_t* __restrict__ assign,
                                              float* __restrict__ best_sim) {
  constexpr int E = elem<T>::per16;
  constexpr int BN = 64 * NT;
  constexpr int ROWS = SIM_BM + BN;
  constexpr int PPT = ROWS / 32;                 // 16-byte pieces a thread moves per step
  constexpr int PPT_A = SIM_BM / 32;             // of which source rows
  constexpr int STAGE = ROWS * SIM_LDSROW;
  extern __shared__ __align__(16) char lds[];
  float* norm2 = reinterpret_cast<float*>(lds + 2 * STAGE);   // [ROWS]
  float* part_v = norm2 + ROWS;                               // [2][BM]
  int* part_c = reinterpret_cast<int*>(part_v + 2 * SIM_BM);  // [2][BM]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, hf = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  const int b = blockIdx.y, m0 = blockIdx.x * SIM_BM;
  const int piece = tid & 7, rbase = tid >> 3;
  const char* xb = reinterpret_cast<const char*>(xv + b * sb);
  const int64_t rowb = sr * (int64_t)sizeof(T);
  const int steps = (D * (int)sizeof(T)) / 128;

  const char* rp[PPT];
#pragma unroll
  for (int i = 0; i < PPT_A; ++i) {
    int r = min(m0 + rbase + 32 * i, M - 1);
    rp[i] = xb + (int64_t)pruned[(int64_t)b * M + r] * rowb + piece * 16;
  }
  float run_v = -INFINITY;   // running best over destination passes (threads < BM)
  int run_c = 0;
  float ss[PPT];
#pragma unroll
  for (int i = 0; i < PPT; ++i) ss[i] = 0.0f;

  const int npass = (k + BN - 1) / BN;
  for (int pass = 0; pass < npass; ++pass) {
    const int n0 = pass * BN;
#pragma unroll
    for (int i = PPT_A; i < PPT; ++i) {
      int c = min(n0 + rbase + 32 * (i - PPT_A), k - 1);
      rp[i] = xb + (int64_t)kept[(int64_t)b * k + c] * rowb + piece * 16;
      ss[i] = 0.0f;
    }
    f32x16_t acc[2][NT];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][t][v] = 0.0f;

    uint4 stg[PPT];
    auto fetch = [&](int s) {
#pragma unroll
      for (int i = 0; i < PPT; ++i) stg[i] = ldg16(rp[i] + (int64_t)s * 128);
    };
    auto stash = [&](int buf, bool count_src) {
      char* dst = lds + buf * STAGE + rbase * SIM_LDSROW + piece * 16;
#pragma unroll
      for (int i = 0; i < PPT; ++i) {
        *reinterpret_cast<uint4*>(dst + i * 32 * SIM_LDSROW) = stg[i];
        if (i >= PPT_A || count_src) {
          float f[E];
          unpack16<T>(stg[i], f);
#pragma unroll
          for (int e = 0; e < E; ++e) ss[i] = fmaf(f[e], f[e], ss[i]);
        }
      }
    };
    fetch(0);
    stash(0, pass == 0);
    __syncthreads();
    for (int s = 0; s < steps; ++s) {
      if (s + 1 < steps) fetch(s + 1);
      const char* A = lds + (s & 1) * STAGE + (wm * 64 + n) * SIM_LDSROW + hf * 64;
      const char* Bp = lds + (s & 1) * STAGE + (SIM_BM + wn * (BN / 2) + n) * SIM_LDSROW + hf * 64;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        uint4 a0 = *reinterpret_cast<const uint4*>(A + kk * 16);
        uint4 a1 = *reinterpret_cast<const uint4*>(A + 32 * SIM_LDSROW + kk * 16);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          uint4 bv = *reinterpret_cast<const uint4*>(Bp + t * 32 * SIM_LDSROW + kk * 16);
          mma32<T>(acc[0][t], a0, bv);
          mma32<T>(acc[1][t], a1, bv);
        }
      }
      if (s + 1 < steps) stash((s + 1) & 1, pass == 0);
      __syncthreads();
    }
    // squared norms: 8 consecutive lanes share a row
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
      float v = ss[i];
      v += __shfl_xor(v, 1);
      v += __shfl_xor(v, 2);
      v += __shfl_xor(v, 4);
      if (piece == 0 && (i >= PPT_A || pass == 0)) norm2[rbase + 32 * i] = v;
    }
    __syncthreads();
    // row arg-max of dot / |x_i| over this pass's destinations (|x_j| > 0 does not move it)
    float invk[NT];
    int colv[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      int cl = wn * (BN / 2) + t * 32 + n;
      colv[t] = n0 + cl;
      invk[t] = 1.0f / fmaxf(sqrtf(norm2[SIM_BM + cl]), 1e-8f);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float bv = -INFINITY;
        int bc = 0x7fffffff;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          float c = acc[i][t][v] * invk[t];
          if (colv[t] < k && c > bv) { bv = c; bc = colv[t]; }
        }
#pragma unroll
        for (int off = 1; off < 32; off <<= 1) {
          float ov = __shfl_xor(bv, off);
          int oc = __shfl_xor(bc, off);
          if (ov > bv || (ov == bv && oc < bc)) { bv = ov; bc = oc; }
        }
        if (n == 0) {
          int row = wm * 64 + i * 32 + mma32_row(v, lane);
          part_v[wn * SIM_BM + row] = bv;
          part_c[wn * SIM_BM + row] = bc;
        }
      }
    __syncthreads();
    if (tid < SIM_BM) {
      float v0 = part_v[tid], v1 = part_v[SIM_BM + tid];
      int c0 = part_c[tid], c1 = part_c[SIM_BM + tid];
      if (v1 > v0 || (v1 == v0 && c1 < c0)) { v0 = v1; c0 = c1; }
      if (v0 > run_v) { run_v = v0; run_c = c0; }     // earlier passes hold smaller columns
    }
    __syncthreads();
  }
  if (tid < SIM_BM && m0 + tid < M) {
    float c = run_v / fmaxf(sqrtf(norm2[tid]), 1e-8f);
    int64_t o = (int64_t)b * M + m0 + tid;
    best_sim[o] = c;
    assign[o] = (c > threshold) ? run_c : -1;
  }
}

// ------------------------------------------------------------------------------------------
// k_merge: grid (P + k + Tmax, B), 256 threads.
// ------------------------------------------------------------------------------------------
constexpr int MERGE_SEG = 2048;   // entries of assign[] scanned per round

template <typename T, int CPT>    // CPT = 16-byte chunks of a row per thread (row = D elements)
__global__ __launch_bounds__(256) void k_merge(const T* __restrict__ hidden, int64_t sb, int64_t sr, int D,
                                                int P, int V, int k, int Tmax, float mu,
                                                const float* __restrict__ s_hat, const int32_t* __restrict__ text_len,
                                                const int32_t* __restrict__ kept, const int32_t* __restrict__ pruned,
                                                const int32_t* __restrict__ assign, T* __restrict__ out,
                                                int32_t* __restrict__ pos_out, int32_t* __restrict__ new_len,
                                                float* __restrict__ wsum, int32_t* __restrict__ final_idx) {
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
    for (int c = tid; c < nchunks; c += 256) *reinterpret_cast<uint4*>(orow + c * 16) = ldg16(s + c * 16);
    return;
  }

  const int slot = nrow - P;
  const int M = V - k;
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
      unpack16<T>(ldg16(xrow + c * 16), f);
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
          if (c < nchunks) ch[u][q] = ldg16(srow + c * 16);
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
        *reinterpret_cast<uint4*>(orow + c * 16) = pack16<T>(f);
      }
    }
  } else {                                               // nothing absorbed: Eq. 6 is the identity
    for (int c = tid; c < nchunks; c += 256) *reinterpret_cast<uint4*>(orow + c * 16) = ldg16(xrow + c * 16);
  }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
template <typename T, int NT>
static hipError_t launch_sim(const asap_params& p, const T* xv, int64_t sb, int64_t sr, const int32_t* pruned,
                             const int32_t* kept, int32_t* assign, float* best_sim, hipStream_t st, Timer* tm) {
  constexpr int BN = 64 * NT, ROWS = SIM_BM + BN;
  const size_t lds = 2 * (size_t)ROWS * SIM_LDSROW + sizeof(float) * ROWS + 4 * sizeof(float) * SIM_BM;
  auto kern = k_sim<T, NT>;
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  const int M = p.V - p.k;
  ASAP_LAUNCH(tm, "k_sim", kern, dim3((M + SIM_BM - 1) / SIM_BM, p.B), dim3(256), lds, st, xv, sb, sr, p.D, pruned,
              kept, M, p.k, p.sim_threshold, assign, best_sim);
  return hipGetLastError();
}

// destination tile width: fewest padded columns overall, then fewest passes
static int pick_nt(int k) {
  int best_nt = 5;
  long best_cost = -1;
  for (int nt = 1; nt <= 5; ++nt) {
    long bn = 64 * nt, passes = (k + bn - 1) / bn;
    long cost = passes * bn * 8 + passes;     // padded MFMA columns dominate
    if (best_cost < 0 || cost < best_cost) { best_cost = cost; best_nt = nt; }
  }
  return best_nt;
}

template <typename T>
static hipError_t merge_typed(const asap_params& p, const void* hidden, int64_t hsb, int64_t hsr,
                              const float* s_hat, const int32_t* text_len, const int32_t* kept,
                              const int32_t* pruned, void* out_hidden, int32_t* pos_out, int32_t* new_len,
                              int32_t* assign, float* best_sim, float* wsum, int32_t* final_idx,
                              hipStream_t st, Timer* tm) {
  const T* h = static_cast<const T*>(hidden);
  hipError_t e = hipSuccess;
  if (p.V > p.k) {
    const T* xv = h + (int64_t)p.P * hsr;
    switch (pick_nt(p.k)) {
      case 1: e = launch_sim<T, 1>(p, xv, hsb, hsr, pruned, kept, assign, best_sim, st, tm); break;
      case 2: e = launch_sim<T, 2>(p, xv, hsb, hsr, pruned, kept, assign, best_sim, st, tm); break;
      case 3: e = launch_sim<T, 3>(p, xv, hsb, hsr, pruned, kept, assign, best_sim, st, tm); break;
      case 4: e = launch_sim<T, 4>(p, xv, hsb, hsr, pruned, kept, assign, best_sim, st, tm); break;
      default: e = launch_sim<T, 5>(p, xv, hsb, hsr, pruned, kept, assign, best_sim, st, tm); break;
    }
    if (e != hipSuccess) return e;
  }
  constexpr int E = elem<T>::per16;
  const int nchunks = p.D / E;
  const int cpt = (nchunks + 255) / 256;
  dim3 grid(p.P + p.k + p.Tmax, p.B);
#define ASAP_MERGE(CPT)                                                                                    \
  ASAP_LAUNCH(tm, "k_merge", (k_merge<T, CPT>), grid, dim3(256), 0, st, h, hsb, hsr, p.D, p.P, p.V, p.k,   \
              p.Tmax, p.merge_weight, s_hat, text_len, kept, pruned, assign, static_cast<T*>(out_hidden),  \
              pos_out, new_len, wsum, final_idx)
  if (cpt <= 1) ASAP_MERGE(1);
  else if (cpt <= 2) ASAP_MERGE(2);
  else if (cpt <= 4) ASAP_MERGE(4);
  else if (cpt <= 8) ASAP_MERGE(8);
  else return hipErrorInvalidValue;
#undef ASAP_MERGE
  return hipGetLastError();
}

hipError_t launch_merge(const asap_params& p, const void* hidden, int64_t hsb, int64_t hsr,
                        const float* s_hat, const int32_t* text_len, const int32_t* kept,
                        const int32_t* pruned, void* out_hidden, int32_t* pos_out, int32_t* new_len,
                        int32_t* assign, float* best_sim, float* wsum, int32_t* final_idx,
                        hipStream_t st, Timer* tm) {
  if (p.h_dtype == ASAP_BF16)
    return merge_typed<bf16_t>(p, hidden, hsb, hsr, s_hat, text_len, kept, pruned, out_hidden, pos_out,
                               new_len, assign, best_sim, wsum, final_idx, st, tm);
  return merge_typed<float>(p, hidden, hsb, hsr, s_hat, text_len, kept, pruned, out_hidden, pos_out, new_len,
                            assign, best_sim, wsum, final_idx, st, tm);
}

}  // namespace asap
