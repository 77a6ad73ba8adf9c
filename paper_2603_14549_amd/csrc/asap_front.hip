// Eq. 2 from hidden states (Sec. 3.1: q_m = R_{Theta,m} W_q x_m): the sum of the visual queries, the
// only thing Eq. 2 needs of them, without any visual query being formed.  The rotation acts on the
// coordinate pairs (c, c + d/2) of every head with the same angle pos * theta^(-2c/d), so
//   sum_i q_i[c]       = w_c . Xc_c - w_{c+d/2} . Xs_c
//   sum_i q_i[c + d/2] = w_{c+d/2} . Xc_c + w_c . Xs_c,        w_e = row e of the head's W_q,
//   Xc_c = sum_i cos(pos_i theta_c) x_i,   Xs_c = sum_i sin(pos_i theta_c) x_i     (vectors of length D)
// and the d trigonometric sums Xc, Xs are shared by all heads.
//
//   k_rope_table   cos / sin of every (visual token, frequency) in fp64, stored as f32 [B, V, d]
//   k_trig_sums    Y[b, r, :] = sum_i table[b, i, r] x_{b,i}: fp32 FMAs on the vector ALUs in runs of 64
//                  tokens, the runs added in fp64; a workgroup = 64 hidden columns x 4 waves of d/4 rows
//   k_qbar_project the 2 x 2 dot products above per (head, frequency, image) -> per-head summed queries
//                  in the layout k_qsum leaves, so that k_qsplit and everything after it run unchanged
// This is the front end as a measured prototype: it reads the visual hidden states, B V D elements,
// where k_qsum reads the visual queries, B H V d elements -- the same bytes whenever H d = D -- and
// adds 2 d V D multiply-adds per image on top, so it cannot be faster than k_qsum.
#include "asap_device.hpp"
#include "asap_launch.hpp"

namespace asap {

// grid (ceil(V / 64), B), 64 threads: thread = one visual token
__global__ __launch_bounds__(64) void k_rope_table(const int32_t* __restrict__ positions, int pos0, int V, int d,
                                                    double log2_theta, float* __restrict__ tab) {
  const int b = blockIdx.y, i = blockIdx.x * 64 + threadIdx.x;
  if (i >= V) return;
  const double pos = positions ? (double)positions[(int64_t)b * V + i] : (double)(pos0 + i);
  float* out = tab + ((int64_t)b * V + i) * d;
  const int half = d / 2;
  for (int c = 0; c < half; ++c) {
    const double ang = pos * exp2(-2.0 * (double)c / (double)d * log2_theta);
    double sn, cs;
    sincos(ang, &sn, &cs);
    out[c] = (float)cs;
    out[half + c] = (float)sn;
  }
}

template <typename T> __device__ __forceinline__ float load_elem(const T* p);
template <> __device__ __forceinline__ float load_elem<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_elem<bf16_t>(const bf16_t* p) { return bf16_bits_to_f32(p->bits); }

// grid (D / 64, B), 256 threads = 4 waves; wave w owns rows [w RPW, (w+1) RPW) of the d table rows,
// lane n the hidden column 64 blockIdx.x + n.  The table row of a token is wave-uniform (scalar loads).
constexpr int FRONT_RUN = 64;      // tokens added in fp32 before the run goes into the fp64 sum
template <typename T, int RPW>
__global__ __launch_bounds__(256) void k_trig_sums(const T* __restrict__ hidden, int64_t sb, int64_t sr, int P, int V,
                                                    int D, const float* __restrict__ tab, float* __restrict__ Y) {
  const int b = blockIdx.y, n = blockIdx.x * 64 + (threadIdx.x & 63);
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int d = 4 * RPW;
  const T* x = hidden + b * sb + (int64_t)P * sr + n;
  const float* t = tab + (int64_t)b * V * d + w * RPW;
  double total[RPW];
  float run[RPW];
#pragma unroll
  for (int r = 0; r < RPW; ++r) { total[r] = 0.0; run[r] = 0.0f; }
  for (int i0 = 0; i0 < V; i0 += FRONT_RUN) {
    const int i1 = min(V, i0 + FRONT_RUN);
    int i = i0;
    for (; i + 3 < i1; i += 4) {       // four tokens in flight
      float xv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) xv[u] = load_elem<T>(x + (int64_t)(i + u) * sr);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float* tr = t + (int64_t)(i + u) * d;
#pragma unroll
        for (int r = 0; r < RPW; ++r) run[r] = fmaf(tr[r], xv[u], run[r]);
      }
    }
    for (; i < i1; ++i) {
      const float xv = load_elem<T>(x + (int64_t)i * sr);
      const float* tr = t + (int64_t)i * d;
#pragma unroll
      for (int r = 0; r < RPW; ++r) run[r] = fmaf(tr[r], xv, run[r]);
    }
#pragma unroll
    for (int r = 0; r < RPW; ++r) { total[r] += (double)run[r]; run[r] = 0.0f; }
  }
  float* out = Y + ((int64_t)b * d + w * RPW) * D + n;
#pragma unroll
  for (int r = 0; r < RPW; ++r) out[(int64_t)r * D] = (float)total[r];
}

// grid (d / 2, H, B), 256 threads.  Rows c and c + d/2 of head h's W_q against Y[b, c] (cos sums) and
// Y[b, d/2 + c] (sin sums): 16 elements per thread and product in fp32, the rest in fp64, fixed order.
// Writes qpart [B, H, 1, d] (the layout of k_qsum with one chunk).
template <typename T>
__global__ __launch_bounds__(256) void k_qbar_project(const T* __restrict__ wq, const float* __restrict__ Y, int H,
                                                       int d, int D, double* __restrict__ qpart) {
  constexpr int E = elem<T>::per16;
  __shared__ double red[4][4];
  const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z, half = d / 2;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const T* w0 = wq + ((int64_t)h * d + c) * D;
  const T* w1 = wq + ((int64_t)h * d + half + c) * D;
  const float* yc = Y + ((int64_t)b * d + c) * D;
  const float* ys = Y + ((int64_t)b * d + half + c) * D;
  double acc[4] = {0.0, 0.0, 0.0, 0.0};       // w0.yc, w1.ys, w1.yc, w0.ys
  for (int q = tid * E; q < D; q += 256 * E) {
    float a[E], bb[E], fc[E], fs[E];
    unpack16<T>(ldg16(w0 + q), a);
    unpack16<T>(ldg16(w1 + q), bb);
#pragma unroll
    for (int e = 0; e < E; e += 4) {
      unpack16<float>(ldg16(yc + q + e), fc + e);
      unpack16<float>(ldg16(ys + q + e), fs + e);
    }
    float p[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int e = 0; e < E; ++e) {
      p[0] = fmaf(a[e], fc[e], p[0]);
      p[1] = fmaf(bb[e], fs[e], p[1]);
      p[2] = fmaf(bb[e], fc[e], p[2]);
      p[3] = fmaf(a[e], fs[e], p[3]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) acc[u] += (double)p[u];
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    double a = acc[u];
    for (int off = 32; off >= 1; off >>= 1) a += shfl_xor_f64(a, off);
    if (lane == 0) red[wave][u] = a;
  }
  __syncthreads();
  if (tid == 0) {
    double s[4];
    for (int u = 0; u < 4; ++u) s[u] = ((red[0][u] + red[1][u]) + red[2][u]) + red[3][u];
    double* out = qpart + ((int64_t)b * H + h) * d;
    out[c] = s[0] - s[1];
    out[half + c] = s[2] + s[3];
  }
}

size_t front_workspace_bytes(const asap_params& p) {
  return align256(sizeof(float) * (size_t)p.B * p.V * p.d) + align256(sizeof(float) * (size_t)p.B * p.d * p.D);
}

// qpart [B, H, 1, d] from the hidden states; ws: front_workspace_bytes(p)
hipError_t launch_front_end(const asap_params& p, const void* hidden, int64_t hsb, int64_t hsr, const void* wq,
                            double rope_theta, const int32_t* vis_positions, double* qpart, char* ws, hipStream_t st,
                            Timer* tm) {
  float* tab = reinterpret_cast<float*>(ws);
  float* Y = reinterpret_cast<float*>(ws + align256(sizeof(float) * (size_t)p.B * p.V * p.d));
  ASAP_LAUNCH(tm, "k_rope_table", k_rope_table, dim3((p.V + 63) / 64, p.B), dim3(64), 0, st, vis_positions, p.P, p.V,
              p.d, log2(rope_theta), tab);
  const dim3 g1(p.D / 64, p.B), g2(p.d / 2, p.H, p.B);
  if (p.h_dtype == ASAP_BF16) {
    const bf16_t* x = static_cast<const bf16_t*>(hidden);
    if (p.d == 128)
      ASAP_LAUNCH(tm, "k_trig_sums", (k_trig_sums<bf16_t, 32>), g1, dim3(256), 0, st, x, hsb, hsr, p.P, p.V, p.D, tab, Y);
    else
      ASAP_LAUNCH(tm, "k_trig_sums", (k_trig_sums<bf16_t, 16>), g1, dim3(256), 0, st, x, hsb, hsr, p.P, p.V, p.D, tab, Y);
    ASAP_LAUNCH(tm, "k_qbar_project", k_qbar_project<bf16_t>, g2, dim3(256), 0, st, static_cast<const bf16_t*>(wq), Y,
                p.H, p.d, p.D, qpart);
  } else {
    const float* x = static_cast<const float*>(hidden);
    if (p.d == 128)
      ASAP_LAUNCH(tm, "k_trig_sums", (k_trig_sums<float, 32>), g1, dim3(256), 0, st, x, hsb, hsr, p.P, p.V, p.D, tab, Y);
    else
      ASAP_LAUNCH(tm, "k_trig_sums", (k_trig_sums<float, 16>), g1, dim3(256), 0, st, x, hsb, hsr, p.P, p.V, p.D, tab, Y);
    ASAP_LAUNCH(tm, "k_qbar_project", k_qbar_project<float>, g2, dim3(256), 0, st, static_cast<const float*>(wq), Y,
                p.H, p.d, p.D, qpart);
  }
  return hipGetLastError();
}

}  // namespace asap
