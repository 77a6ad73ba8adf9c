// asap_attention: the attention forward of one decoder layer in front of the pruning layer under the
// salience-guided bidirectional mask (Eq. 4-5 on the whole sequence; Eq. 1 with the mask off):
//   out[b,h,i,:] = sum_j A_ij v[b,g(h),j,:],  A_i. = softmax_j( q_i.k_j / sqrt(d) + M_ij ),
//   M_ij = 0 (j <= i);  ln(max(lambda_max s_hat_j, eps)) (j > i, both inside the image span);  -inf otherwise.
// Flash-style: one pass over the keys with running row maxima and sums, both contractions on the
// matrix cores, nothing of size N x N ever stored.
//
//   k_att_bias      log2 of the per-key discount, [B,V]
//   k_vtranspose    values transposed per (image, kv head) to [d, Npad]: the second contraction wants
//                   its A operand (a row of values^T) contiguous along the keys
//   k_attention     grid (ceil(N/128), H, B), 256 threads = 4 waves of 32 queries.  Per 32-key tile a
//                   wave computes S^T = K_tile Q^T (keys are the tile rows, so lane l owns query l % 32
//                   and holds 16 of the tile's keys: the softmax bookkeeping is per lane), then
//                   O^T += V^T_tile P^T, where the P^T operand is taken straight from the accumulator
//                   registers: the contraction slice a lane half supplies is defined as the keys that
//                   lane half already holds, and the V^T operand is loaded to match.
#include "asap_device.hpp"
#include "asap_launch.hpp"

namespace asap {

__global__ __launch_bounds__(256) void k_att_bias(const float* __restrict__ s_hat, int n, float lambda_max, float eps,
                                                   float* __restrict__ bias2) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) bias2[i] = log2f(fmaxf(lambda_max * s_hat[i], eps));
}

// grid (ceil(Npad/32), Hkv, B), 256 threads; vt[b,g,c,n] = v[b,g,n,c] for n < N, 0 for N <= n < Npad
template <typename T>
__global__ __launch_bounds__(256) void k_vtranspose(const T* __restrict__ v, Strides3 sv, int N, int Npad, int d,
                                                     T* __restrict__ vt) {
  __shared__ T tile[32][129];
  const int n0 = blockIdx.x * 32, g = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  const T* src = v + b * sv.b + g * sv.h;
  for (int idx = tid; idx < 32 * d; idx += 256) {
    const int r = idx / d, c = idx - r * d;
    T x{};
    if (n0 + r < N) x = src[(int64_t)(n0 + r) * sv.r + c];
    tile[r][c] = x;
  }
  __syncthreads();
  T* dst = vt + ((int64_t)b * gridDim.y + g) * d * Npad;
  for (int idx = tid; idx < 32 * d; idx += 256) {
    const int c = idx >> 5, r = idx & 31;
    dst[(int64_t)c * Npad + n0 + r] = tile[r][c];
  }
}

__device__ __forceinline__ float fast_exp2_att(float x) { return __builtin_amdgcn_exp2f(x); }

// four consecutive output elements from floats (one rounding to the storage type)
template <typename T> __device__ __forceinline__ void store4(T* dst, const float* f);
template <> __device__ __forceinline__ void store4<float>(float* dst, const float* f) {
  *reinterpret_cast<uint4*>(dst) = pack16<float>(f);
}
template <> __device__ __forceinline__ void store4<bf16_t>(bf16_t* dst, const float* f) {
  *reinterpret_cast<uint2*>(dst) =
      make_uint2(f32_to_bf16_bits(f[0]) | (f32_to_bf16_bits(f[1]) << 16), f32_to_bf16_bits(f[2]) | (f32_to_bf16_bits(f[3]) << 16));
}

// key held in accumulator register v of a lane of half hf, relative to the tile
__device__ __forceinline__ int att_key_of(int v, int hf) { return 8 * (v >> 2) + 4 * hf + (v & 3); }

template <typename T, int CH>   // CH = 16-byte chunks of a row per lane half (row bytes = 32 * CH)
__global__ __launch_bounds__(256) void k_attention(const T* __restrict__ q, Strides3 sq, const T* __restrict__ k,
                                                    Strides3 sk, const T* __restrict__ vt, int Npad,
                                                    const float* __restrict__ bias2, T* __restrict__ out, int H,
                                                    int Hkv, int N, int P, int V, float c2) {
  constexpr int E = elem<T>::per16;            // elements per 16-byte chunk
  constexpr int D = CH * 2 * E;                // head dimension
  constexpr int DT = D / 32;                   // 32-row tiles of O^T
  constexpr int NPS = 32 / (2 * E);            // contraction steps of the second product per key tile
  constexpr int GPC = E / 4;                   // groups of 4 consecutive keys in a lane's chunk
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, hf = lane >> 5;
  const int b = blockIdx.z, h = blockIdx.y, g = (h * Hkv) / H;
  const int i0 = blockIdx.x * 128 + wave * 32;
  if (i0 >= N) return;
  const int i = i0 + n, i_ld = min(i, N - 1);
  const int i_hi = min(i0 + 31, N - 1);
  const bool bidir = bias2 != nullptr;
  const int img_lo = P, img_hi = P + V;         // image span [img_lo, img_hi)
  const bool q_img = bidir && i >= img_lo && i < img_hi;

  // queries: B operand of S^T, pieces 2c + hf of the row
  uint4 qa[CH];
  {
    const char* qrow = reinterpret_cast<const char*>(q + b * sq.b + h * sq.h + (int64_t)i_ld * sq.r) + hf * 16;
#pragma unroll
    for (int c = 0; c < CH; ++c) qa[c] = ldg16(qrow + c * 32);
  }
  const char* kbase = reinterpret_cast<const char*>(k + b * sk.b + g * sk.h) + hf * 16;
  const int64_t krow_bytes = sk.r * (int64_t)sizeof(T);
  // values^T: lane (m, hf) reads row t*32 + m, the keys its partner lanes hold
  const char* vbase = reinterpret_cast<const char*>(vt + (((int64_t)b * Hkv + g) * D + n) * Npad) + 4 * hf * sizeof(T);
  const int64_t vtile_bytes = (int64_t)32 * Npad * sizeof(T);

  f32x16_t o[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[t][v] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;

  // keys this wave has to visit: up to its last query, or to the end of the image span if it holds
  // image rows (their future image keys count, discounted)
  int j_last = i_hi;
  if (bidir && i_hi >= img_lo && i0 < img_hi) j_last = max(j_last, img_hi - 1);

  for (int j0 = 0; j0 <= j_last; j0 += 32) {
    uint4 kb[CH];
    {
      const char* krow = kbase + (int64_t)min(j0 + n, N - 1) * krow_bytes;
#pragma unroll
      for (int c = 0; c < CH; ++c) kb[c] = ldg16(krow + c * 32);
    }
    uint4 va[DT][NPS];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int c = 0; c < NPS; ++c) {
        const char* p0 = vbase + t * vtile_bytes + (int64_t)(j0 + 8 * c * GPC) * sizeof(T);
        if (GPC == 1) {
          va[t][c] = ldg16(p0);                          // 4 keys of 4 bytes
        } else {
          const uint2 lo = *reinterpret_cast<const uint2*>(p0);                       // keys +0..3
          const uint2 hi = *reinterpret_cast<const uint2*>(p0 + 8 * sizeof(T));       // keys +8..11
          va[t][c] = make_uint4(lo.x, lo.y, hi.x, hi.y);
        }
      }
    f32x16_t s;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.0f;
#pragma unroll
    for (int c = 0; c < CH; ++c) mma32<T>(s, kb[c], qa[c]);

    float z[16];
    const bool plain = j0 + 31 <= i0;          // every key of the tile precedes every query of the wave
    if (plain) {
#pragma unroll
      for (int v = 0; v < 16; ++v) z[v] = s[v] * c2;
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int j = j0 + att_key_of(v, hf);
        float mb = -INFINITY;
        if (j < N) {
          if (j <= i) mb = 0.0f;
          else if (q_img && j >= img_lo && j < img_hi) mb = bias2[(int64_t)b * V + (j - img_lo)];
        }
        z[v] = s[v] * c2 + mb;
      }
    }
    float mx = z[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) mx = fmaxf(mx, z[v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);       // finite from the first tile on: key 0 precedes every query
    const float alpha = fast_exp2_att(m_run - m_new);
    float p[16], psum = 0.0f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      p[v] = fast_exp2_att(z[v] - m_new);
      psum += p[v];
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[t][v] *= alpha;
#pragma unroll
    for (int c = 0; c < NPS; ++c) {
      const uint4 pb = pack16<T>(&p[c * E]);
#pragma unroll
      for (int t = 0; t < DT; ++t) mma32<T>(o[t], va[t][c], pb);
    }
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = 1.0f / l_tot;
  if (i < N) {
    T* orow = out + (((int64_t)b * H + h) * N + i) * D;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        float f[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) f[e] = o[t][4 * gq + e] * inv;
        store4<T>(orow + t * 32 + 8 * gq + 4 * hf, f);
      }
  }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
static int att_npad(const asap_params& p) { return ((p.P + p.V + p.Tmax + 31) / 32) * 32 + 32; }

size_t attention_workspace_bytes(const asap_params& p) {
  const size_t es = p.qk_dtype == ASAP_BF16 ? 2 : 4;
  return align256(es * (size_t)p.B * p.Hkv * p.d * att_npad(p)) + align256(sizeof(float) * (size_t)p.B * p.V);
}

template <typename T>
static hipError_t attention_typed(const asap_params& p, const void* q, Strides3 sq, const void* k, Strides3 sk,
                                  const void* v, Strides3 sv, const float* s_hat, void* out, char* ws,
                                  hipStream_t st, Timer* tm) {
  constexpr int E = elem<T>::per16;
  const int N = p.P + p.V + p.Tmax, Npad = att_npad(p);
  T* vt = reinterpret_cast<T*>(ws);
  float* bias2 = reinterpret_cast<float*>(ws + align256(sizeof(T) * (size_t)p.B * p.Hkv * p.d * Npad));
  const bool bidir = p.mask_mode == ASAP_MASK_KEYBIAS;
  if (bidir)
    ASAP_LAUNCH(tm, "k_att_bias", k_att_bias, dim3((p.B * p.V + 255) / 256), dim3(256), 0, st, s_hat, p.B * p.V,
                p.lambda_max, p.eps, bias2);
  ASAP_LAUNCH(tm, "k_vtranspose", k_vtranspose<T>, dim3(Npad / 32, p.Hkv, p.B), dim3(256), 0, st,
              static_cast<const T*>(v), sv, N, Npad, p.d, vt);
  const float c2 = 1.4426950408889634f / sqrtf((float)p.d);
  const dim3 grid((N + 127) / 128, p.H, p.B);
  const int ch = p.d / E / 2;
#define ASAP_ATT(CHV)                                                                                          \
  ASAP_LAUNCH(tm, "k_attention", (k_attention<T, CHV>), grid, dim3(256), 0, st, static_cast<const T*>(q), sq,   \
              static_cast<const T*>(k), sk, vt, Npad, bidir ? bias2 : nullptr, static_cast<T*>(out), p.H, p.Hkv, \
              N, p.P, p.V, c2)
  if (ch == 4) ASAP_ATT(4);
  else if (ch == 8) ASAP_ATT(8);
  else if (ch == 16) ASAP_ATT(16);
  else return hipErrorInvalidValue;
#undef ASAP_ATT
  return hipGetLastError();
}

hipError_t launch_attention(const asap_params& p, const void* q, Strides3 sq, const void* k, Strides3 sk,
                            const void* v, Strides3 sv, const float* s_hat, void* out, char* ws, hipStream_t st,
                            Timer* tm) {
  if (p.qk_dtype == ASAP_BF16) return attention_typed<bf16_t>(p, q, sq, k, sk, v, sv, s_hat, out, ws, st, tm);
  return attention_typed<float>(p, q, sq, k, sk, v, sv, s_hat, out, ws, st, tm);
}

}  // namespace asap
