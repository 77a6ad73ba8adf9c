// asap_score: Eq. 2 (raw attention mass), Eq. 3 (salience), Eq. 4 (discount) and the text-row
// softmax of Eq. 5 reduced to one selection score per visual token.
//
// Kernels, in launch order:
//   k_qsum      column sums of the visual queries, per (image, head, row chunk), fp64
//   k_qbar      fixed-order sum of those partials per kv head
//   k_mass      s_j = sum_g qbar_g . k_{g,j} / (H sqrt d)        (Eq. 2 by linearity), fp64
//   k_salience  min / max per image, s_hat (Eq. 3), lambda' (Eq. 4)
//   k_text_attn per (image, head): text-query x visual-key logits on the matrix cores, two
//               sweeps over the keys (row statistics, then normalised column sums)
//   k_score     fixed-order head reduction, times lambda', mean over heads and text rows, fp64
#include "asap_device.hpp"
#include "asap_launch.hpp"

namespace asap {

// ------------------------------------------------------------------------------------------
// k_qsum: grid (q_chunks, H, B), 256 threads.  Rows are d elements = LPR 16-byte pieces; a
// thread keeps the piece tid % LPR of rows tid / LPR, tid / LPR + RPI, ...
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_qsum(const T* __restrict__ q, Strides3 sq, int V, int d, int R,
                                               double* __restrict__ qpart) {
  constexpr int E = elem<T>::per16;
  const int LPR = d / E, RPI = 256 / LPR;
  const int tid = threadIdx.x, piece = tid % LPR, r0 = tid / LPR;
  const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int lo = c * R, hi = min(V, lo + R);
  const T* base = q + b * sq.b + h * sq.h + piece * E;
  double acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.0;
#pragma unroll 4
  for (int row = lo + r0; row < hi; row += RPI) {
    uint4 ch = ldg16(base + (int64_t)row * sq.r);
    float f[E];
    unpack16<T>(ch, f);
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] += (double)f[e];
  }
  __shared__ double red[256 * 8];
#pragma unroll
  for (int e = 0; e < E; ++e) red[r0 * d + piece * E + e] = acc[e];
  __syncthreads();
  if (tid < d) {
    double s = 0.0;
    for (int r = 0; r < RPI; ++r) s += red[r * d + tid];
    qpart[(((int64_t)b * gridDim.y + h) * gridDim.x + c) * d + tid] = s;
  }
}

// k_qbar: grid (Hkv, B), d threads.  qbar[b,g,:] = sum over the heads of group g and chunks.
__global__ void k_qbar(const double* __restrict__ qpart, double* __restrict__ qbar, int H, int Hkv,
                       int nchunk, int d) {
  const int g = blockIdx.x, b = blockIdx.y, c = threadIdx.x;
  const int G = H / Hkv;
  double s = 0.0;
  for (int h = g * G; h < (g + 1) * G; ++h)
    for (int ch = 0; ch < nchunk; ++ch) s += qpart[(((int64_t)b * H + h) * nchunk + ch) * d + c];
  qbar[((int64_t)b * Hkv + g) * d + c] = s;
}

// ------------------------------------------------------------------------------------------
// k_mass: grid (ceil(V/32), B), 256 threads, dynamic LDS = Hkv*d doubles (qbar of the image).
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_mass(const T* __restrict__ kv, Strides3 sk, const double* __restrict__ qbar,
                                               int Hkv, int V, int d, double scale,
                                               double* __restrict__ s64, float* __restrict__ s_raw) {
  constexpr int E = elem<T>::per16;
  constexpr int JT = 32;
  extern __shared__ double qb_s[];
  const int LPR = d / E, RPI = 256 / LPR, NP = JT / RPI;   // NP passes of RPI rows
  const int tid = threadIdx.x, piece = tid % LPR, r0 = tid / LPR;
  const int b = blockIdx.y, j0 = blockIdx.x * JT;
  for (int i = tid; i < Hkv * d; i += 256) qb_s[i] = qbar[(int64_t)b * Hkv * d + i];
  __syncthreads();
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  const T* base = kv + b * sk.b + piece * E;
#pragma unroll 2
  for (int g = 0; g < Hkv; ++g) {
    double qb[E];
#pragma unroll
    for (int e = 0; e < E; ++e) qb[e] = qb_s[g * d + piece * E + e];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      if (p < NP) {
        int row = j0 + p * RPI + r0;
        if (row < V) {
          uint4 ch = ldg16(base + g * sk.h + (int64_t)row * sk.r);
          float f[E];
          unpack16<T>(ch, f);
#pragma unroll
          for (int e = 0; e < E; ++e) acc[p] = fma(qb[e], (double)f[e], acc[p]);
        }
      }
    }
  }
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    if (p < NP) {
      double a = acc[p];
      for (int off = LPR >> 1; off > 0; off >>= 1) a += shfl_xor_f64(a, off);
      int row = j0 + p * RPI + r0;
      if (piece == 0 && row < V) {
        double s = a * scale;
        s64[(int64_t)b * V + row] = s;
        s_raw[(int64_t)b * V + row] = (float)s;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// k_salience: grid (B), 1024 threads.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_salience(const double* __restrict__ s64, int V, double lambda_max,
                                                    double eps, int mask_on, double* __restrict__ mm,
                                                    float* __restrict__ s_hat, float* __restrict__ lam) {
  __shared__ double smin[16], smax[16];
  const int b = blockIdx.x, tid = threadIdx.x;
  const double* s = s64 + (int64_t)b * V;
  double lo = INFINITY, hi = -INFINITY;
  for (int j = tid; j < V; j += 1024) {
    double v = s[j];
    lo = fmin(lo, v);
    hi = fmax(hi, v);
  }
  for (int off = 32; off > 0; off >>= 1) {
    lo = fmin(lo, shfl_xor_f64(lo, off));
    hi = fmax(hi, shfl_xor_f64(hi, off));
  }
  if ((tid & 63) == 0) { smin[tid >> 6] = lo; smax[tid >> 6] = hi; }
  __syncthreads();
  lo = smin[0]; hi = smax[0];
  for (int w = 1; w < 16; ++w) { lo = fmin(lo, smin[w]); hi = fmax(hi, smax[w]); }
  if (tid == 0) { mm[2 * b] = lo; mm[2 * b + 1] = hi; }
  const double inv = 1.0 / (hi - lo + eps);
  for (int j = tid; j < V; j += 1024) {
    double sh = (s[j] - lo) * inv;
    s_hat[(int64_t)b * V + j] = (float)sh;
    lam[(int64_t)b * V + j] = mask_on ? (float)fmax(lambda_max * sh, eps) : 1.0f;
  }
}

// ------------------------------------------------------------------------------------------
// k_text_attn<T, RB, CH>: grid (H, B), 256 threads = 4 waves.
//   RB = 32-row blocks of text queries (Tmax <= 32*RB), CH = 16-byte chunks of a row per lane
//   half (row bytes = 32*CH).  The text queries sit in LDS as MFMA A operands; every wave
//   streams its own 32-key tiles straight from global memory as B operands: lane (n, hf) of
//   a tile reads the half row [hf*16*CH, +16*CH) bytes of key n, the A side reads the same
//   half of its query row, so a chunk pair covers the same contraction slice.
// Sweep 1 keeps, per lane and query row, an online (max, sum) of lambda'_j 2^(z) over the
// keys that lane saw; they are merged across lanes and waves into row max m_t and 1/den_t.
// Sweep 2 recomputes the logits and adds 2^(z - m_t)/den_t over the valid rows into
// upart[b,h,j] (lambda'_j is applied later in fp64).  Logits are kept in log2 units.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int CH>
__device__ __forceinline__ void load_key_tile(uint4 (&kb)[CH], const char* krow) {
#pragma unroll
  for (int c = 0; c < CH; ++c) kb[c] = ldg16(krow + c * 16);
}

template <typename T, int RB, int CH>
__global__ __launch_bounds__(256) void k_text_attn(const T* __restrict__ qt, Strides3 sq, const T* __restrict__ kv,
                                                    Strides3 sk, const float* __restrict__ lam,
                                                    const int32_t* __restrict__ text_len,
                                                    const float* __restrict__ lse_extra, float* __restrict__ upart,
                                                    int H, int Hkv, int V, int Tmax, float scale_hi, float scale_lo) {
  constexpr int ROWB = CH * 32;        // bytes of one query / key row
  constexpr int LDSROW = ROWB + 16;    // padded LDS row
  constexpr int NR = RB * 32;
  constexpr float NEG = -1e30f;
  extern __shared__ __align__(16) char lds[];
  char* q_s = lds;                                              // [NR][LDSROW]
  float* st_m = reinterpret_cast<float*>(lds + NR * LDSROW);    // [4][NR]
  float* st_s = st_m + 4 * NR;                                  // [4][NR]
  float* fin_m = st_s + 4 * NR;                                 // [NR]
  float* fin_i = fin_m + NR;                                    // [NR]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, hf = lane >> 5;
  const int h = blockIdx.x, b = blockIdx.y;
  const int g = (h * Hkv) / H;
  const int len = text_len[b];

  // stage the text queries (rows >= Tmax are zero)
  {
    const char* qbase = reinterpret_cast<const char*>(qt + b * sq.b + h * sq.h);
    constexpr int PPR = ROWB / 16;
    for (int i = tid; i < NR * PPR; i += 256) {
      int row = i / PPR, pc = i % PPR;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (row < Tmax) v = ldg16(qbase + (int64_t)row * sq.r * sizeof(T) + pc * 16);
      *reinterpret_cast<uint4*>(q_s + row * LDSROW + pc * 16) = v;
    }
  }
  __syncthreads();

  const char* kbase = reinterpret_cast<const char*>(kv + b * sk.b + g * sk.h) + hf * (CH * 16);
  const int64_t krow_bytes = sk.r * (int64_t)sizeof(T);
  const float* lam_b = lam + (int64_t)b * V;
  const int ntiles = (V + 31) >> 5;
  const char* qa = q_s + n * LDSROW + hf * (CH * 16);

  float m_run[RB][16], s_run[RB][16];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int v = 0; v < 16; ++v) { m_run[rb][v] = NEG; s_run[rb][v] = 0.0f; }

  // ---------------- sweep 1: row statistics ----------------
  {
    uint4 kb[CH], kn[CH];
    int tile = wave;
    if (tile < ntiles) load_key_tile<CH>(kb, kbase + (int64_t)min(tile * 32 + n, V - 1) * krow_bytes);
    for (; tile < ntiles; tile += 4) {
      const int j = tile * 32 + n;
      const int tnext = tile + 4;
      if (tnext < ntiles) load_key_tile<CH>(kn, kbase + (int64_t)min(tnext * 32 + n, V - 1) * krow_bytes);
      const bool valid = j < V;
      const float lj = valid ? lam_b[j] : 0.0f;
      f32x16_t acc[RB];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[rb][v] = 0.0f;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          uint4 a = *reinterpret_cast<const uint4*>(qa + rb * 32 * LDSROW + c * 16);
          mma32<T>(acc[rb], a, kb[c]);
        }
      }
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float z = fmaf(acc[rb][v], scale_lo, acc[rb][v] * scale_hi);
          z = valid ? z : NEG;
          float dl = z - m_run[rb][v];
          float e = fast_exp2(-fabsf(dl));
          bool gt = dl > 0.0f;
          s_run[rb][v] = fmaf(gt ? s_run[rb][v] : lj, e, gt ? lj : s_run[rb][v]);
          m_run[rb][v] = fmaxf(m_run[rb][v], z);
        }
      if (tnext < ntiles) {
#pragma unroll
        for (int c = 0; c < CH; ++c) kb[c] = kn[c];
      }
    }
  }
  // merge the 32 lanes of a half (they hold the same rows, different keys)
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      float m = m_run[rb][v], s = s_run[rb][v];
#pragma unroll
      for (int off = 1; off < 32; off <<= 1) {
        float m2 = __shfl_xor(m, off), s2 = __shfl_xor(s, off);
        float M = fmaxf(m, m2);
        s = s * fast_exp2(m - M) + s2 * fast_exp2(m2 - M);
        m = M;
      }
      if (n == 0) {
        int row = rb * 32 + mma32_row(v, lane);
        st_m[wave * NR + row] = m;
        st_s[wave * NR + row] = s;
      }
    }
  __syncthreads();
  if (tid < NR) {
    float m = st_m[tid], s = st_s[tid];
    for (int w = 1; w < 4; ++w) {
      float m2 = st_m[w * NR + tid], s2 = st_s[w * NR + tid];
      float M = fmaxf(m, m2);
      s = s * fast_exp2(m - M) + s2 * fast_exp2(m2 - M);
      m = M;
    }
    if (lse_extra != nullptr && tid < Tmax) {
      float l2 = lse_extra[((int64_t)b * H + h) * Tmax + tid] * 1.4426950408889634f;
      float M = fmaxf(m, l2);
      s = s * fast_exp2(m - M) + fast_exp2(l2 - M);
      m = M;
    }
    const bool row_ok = tid < len;
    fin_m[tid] = row_ok ? m : INFINITY;     // 2^(z - inf) = 0: padded rows add nothing
    fin_i[tid] = row_ok ? 1.0f / s : 0.0f;
  }
  __syncthreads();
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      int row = rb * 32 + mma32_row(v, lane);
      m_run[rb][v] = fin_m[row];
      s_run[rb][v] = fin_i[row];
    }

  // ---------------- sweep 2: normalised column sums ----------------
  {
    float* out = upart + ((int64_t)b * H + h) * V;
    uint4 kb[CH], kn[CH];
    int tile = wave;
    if (tile < ntiles) load_key_tile<CH>(kb, kbase + (int64_t)min(tile * 32 + n, V - 1) * krow_bytes);
    for (; tile < ntiles; tile += 4) {
      const int j = tile * 32 + n;
      const int tnext = tile + 4;
      if (tnext < ntiles) load_key_tile<CH>(kn, kbase + (int64_t)min(tnext * 32 + n, V - 1) * krow_bytes);
      f32x16_t acc[RB];
      float u = 0.0f;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[rb][v] = 0.0f;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          uint4 a = *reinterpret_cast<const uint4*>(qa + rb * 32 * LDSROW + c * 16);
          mma32<T>(acc[rb], a, kb[c]);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float z = fmaf(acc[rb][v], scale_lo, acc[rb][v] * scale_hi);
          u = fmaf(fast_exp2(z - m_run[rb][v]), s_run[rb][v], u);
        }
      }
      u += __shfl_xor(u, 32);
      if (hf == 0 && j < V) out[j] = u;
      if (tnext < ntiles) {
#pragma unroll
        for (int c = 0; c < CH; ++c) kb[c] = kn[c];
      }
    }
  }
}

// k_score: grid (ceil(V/256), B), 256 threads.
__global__ __launch_bounds__(256) void k_score(const float* __restrict__ upart, const double* __restrict__ s64,
                                                const double* __restrict__ mm, const int32_t* __restrict__ text_len,
                                                int H, int V, double lambda_max, double eps, int mask_on,
                                                float* __restrict__ score) {
  const int b = blockIdx.y, j = blockIdx.x * 256 + threadIdx.x;
  if (j >= V) return;
  double u = 0.0;
  for (int h = 0; h < H; ++h) u += (double)upart[((int64_t)b * H + h) * V + j];
  double lam = 1.0;
  if (mask_on) {
    double lo = mm[2 * b], hi = mm[2 * b + 1];
    lam = fmax(lambda_max * ((s64[(int64_t)b * V + j] - lo) / (hi - lo + eps)), eps);
  }
  score[(int64_t)b * V + j] = (float)(lam * u / ((double)H * (double)text_len[b]));
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
ScoreWorkspace score_workspace(const asap_params& p) {
  ScoreWorkspace w;
  w.q_rows = 256;
  if ((int64_t)p.B * p.H * ((p.V + 255) / 256) < 1024) w.q_rows = 64;
  w.q_chunks = (p.V + w.q_rows - 1) / w.q_rows;
  size_t off = 0;
  w.off_qpart = off; off = align256(off + sizeof(double) * p.B * p.H * w.q_chunks * p.d);
  w.off_qbar = off;  off = align256(off + sizeof(double) * p.B * p.Hkv * p.d);
  w.off_s64 = off;   off = align256(off + sizeof(double) * p.B * p.V);
  w.off_mm = off;    off = align256(off + sizeof(double) * p.B * 2);
  w.off_lam = off;   off = align256(off + sizeof(float) * p.B * p.V);
  w.off_upart = off; off = align256(off + sizeof(float) * (size_t)p.B * p.H * p.V);
  w.total = off;
  return w;
}

template <typename T, int RB, int CH>
static hipError_t launch_text_attn(const asap_params& p, const void* q_txt, Strides3 qt, const void* k_vis,
                                   Strides3 kv, const float* lam, const int32_t* text_len,
                                   const float* lse_extra, float* upart, hipStream_t st, Timer* tm) {
  constexpr int NR = RB * 32;
  size_t lds = (size_t)NR * (CH * 32 + 16) + sizeof(float) * (10 * NR);
  auto kern = k_text_attn<T, RB, CH>;
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  const double sc = 1.4426950408889634 / sqrt((double)p.d);
  const float hi = (float)sc, lo = (float)(sc - (double)hi);
  ASAP_LAUNCH(tm, "k_text_attn", kern, dim3(p.H, p.B), dim3(256), lds, st, static_cast<const T*>(q_txt), qt,
              static_cast<const T*>(k_vis), kv, lam, text_len, lse_extra, upart, p.H, p.Hkv, p.V, p.Tmax, hi, lo);
  return hipGetLastError();
}

template <typename T, int CH>
static hipError_t dispatch_rb(const asap_params& p, const void* q_txt, Strides3 qt, const void* k_vis,
                              Strides3 kv, const float* lam, const int32_t* text_len, const float* lse_extra,
                              float* upart, hipStream_t st, Timer* tm) {
  switch ((p.Tmax + 31) / 32) {
    case 1: return launch_text_attn<T, 1, CH>(p, q_txt, qt, k_vis, kv, lam, text_len, lse_extra, upart, st, tm);
    case 2: return launch_text_attn<T, 2, CH>(p, q_txt, qt, k_vis, kv, lam, text_len, lse_extra, upart, st, tm);
    case 3: return launch_text_attn<T, 3, CH>(p, q_txt, qt, k_vis, kv, lam, text_len, lse_extra, upart, st, tm);
    case 4: return launch_text_attn<T, 4, CH>(p, q_txt, qt, k_vis, kv, lam, text_len, lse_extra, upart, st, tm);
  }
  return hipErrorInvalidValue;
}

template <typename T>
static hipError_t score_typed(const asap_params& p, const void* q_vis, Strides3 qv, const void* q_txt,
                              Strides3 qt, const void* k_vis, Strides3 kv, const int32_t* text_len,
                              const float* lse_extra, float* s_raw, float* s_hat, float* score, char* ws,
                              hipStream_t st, Timer* tm) {
  const ScoreWorkspace w = score_workspace(p);
  double* qpart = reinterpret_cast<double*>(ws + w.off_qpart);
  double* qbar = reinterpret_cast<double*>(ws + w.off_qbar);
  double* s64 = reinterpret_cast<double*>(ws + w.off_s64);
  double* mm = reinterpret_cast<double*>(ws + w.off_mm);
  float* lam = reinterpret_cast<float*>(ws + w.off_lam);
  float* upart = reinterpret_cast<float*>(ws + w.off_upart);
  const int mask_on = p.mask_mode == ASAP_MASK_KEYBIAS;

  ASAP_LAUNCH(tm, "k_qsum", k_qsum<T>, dim3(w.q_chunks, p.H, p.B), dim3(256), 0, st, static_cast<const T*>(q_vis),
              qv, p.V, p.d, w.q_rows, qpart);
  ASAP_LAUNCH(tm, "k_qbar", k_qbar, dim3(p.Hkv, p.B), dim3(p.d), 0, st, qpart, qbar, p.H, p.Hkv, w.q_chunks, p.d);
  const double scale = 1.0 / ((double)p.H * sqrt((double)p.d));
  ASAP_LAUNCH(tm, "k_mass", k_mass<T>, dim3((p.V + 31) / 32, p.B), dim3(256), sizeof(double) * p.Hkv * p.d, st,
              static_cast<const T*>(k_vis), kv, qbar, p.Hkv, p.V, p.d, scale, s64, s_raw);
  ASAP_LAUNCH(tm, "k_salience", k_salience, dim3(p.B), dim3(1024), 0, st, s64, p.V, (double)p.lambda_max,
              (double)p.eps, mask_on, mm, s_hat, lam);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  constexpr int E = elem<T>::per16;
  const int ch = p.d / E / 2;   // 16-byte chunks per half row
  if (ch == 4) {
    if constexpr (E == 8) e = dispatch_rb<T, 4>(p, q_txt, qt, k_vis, kv, lam, text_len, lse_extra, upart, st, tm);
    else e = hipErrorInvalidValue;
  } else if (ch == 8) {
    e = dispatch_rb<T, 8>(p, q_txt, qt, k_vis, kv, lam, text_len, lse_extra, upart, st, tm);
  } else if (ch == 16) {
    if constexpr (E == 4) e = dispatch_rb<T, 16>(p, q_txt, qt, k_vis, kv, lam, text_len, lse_extra, upart, st, tm);
    else e = hipErrorInvalidValue;
  } else {
    e = hipErrorInvalidValue;
  }
  if (e != hipSuccess) return e;
  ASAP_LAUNCH(tm, "k_score", k_score, dim3((p.V + 255) / 256, p.B), dim3(256), 0, st, upart, s64, mm, text_len,
              p.H, p.V, (double)p.lambda_max, (double)p.eps, mask_on, score);
  return hipGetLastError();
}

hipError_t launch_score(const asap_params& p, const void* q_vis, Strides3 qv, const void* q_txt, Strides3 qt,
                        const void* k_vis, Strides3 kv, const int32_t* text_len, const float* lse_extra,
                        float* s_raw, float* s_hat, float* score, char* ws, hipStream_t st, Timer* tm) {
  if (p.qk_dtype == ASAP_BF16)
    return score_typed<bf16_t>(p, q_vis, qv, q_txt, qt, k_vis, kv, text_len, lse_extra, s_raw, s_hat, score,
                               ws, st, tm);
  return score_typed<float>(p, q_vis, qv, q_txt, qt, k_vis, kv, text_len, lse_extra, s_raw, s_hat, score, ws,
                            st, tm);
}

}  // namespace asap
