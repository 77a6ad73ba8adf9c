// asap_attention: the attention forward of one decoder layer in front of the pruning layer under the
// salience-guided bidirectional mask (Eq. 4-5 on the whole sequence; Eq. 1 with the mask off):
//   out[b,h,i,:] = sum_j A_ij v[b,g(h),j,:],  A_i. = softmax_j( q_i.k_j / sqrt(d) + M_ij ),
//   M_ij = 0 (j <= i);  ln(max(lambda_max s_hat_j, eps)) (j > i, both inside the image span);  -inf otherwise.
// Flash-style: one pass over the keys with running row maxima and sums, both contractions on the
// matrix cores, nothing of size N x N ever stored.
//
//   k_att_bias      log2 of the per-key discount by sequence position, [B,Npad] (-inf off the image span)
//   k_vtranspose    values transposed per (image, kv head) to [d, Npad]: the second contraction wants
//                   its A operand (a row of values^T) contiguous along the keys
//   k_attention     grid (ceil(N/256), H, B), 256 threads = 4 waves of 64 queries (two 32-query blocks,
//                   so that every operand read from LDS feeds two MFMAs).  The 32-key tile of K and
//                   of V^T goes to LDS by direct global -> LDS loads, double buffered, once for the
//                   four waves.  Per tile a wave computes S^T = K_tile Q^T (keys are the tile rows, so
//                   lane l owns query l % 32 and holds 16 of the tile's keys: the softmax bookkeeping
//                   is per lane), then O^T += V^T_tile P^T, where the P^T operand is taken straight
//                   from the accumulator registers: the contraction slice a lane half supplies is
//                   defined as the keys that lane half already holds, and the V^T operand is read to
//                   match.
#include "asap_device.hpp"
#include "asap_launch.hpp"

namespace asap {

// grid (ceil(Npad/256), B): bias2[b,j] by sequence position j: the log2 discount of an image key,
// -inf for every other position (prefix, text, padding)
__global__ __launch_bounds__(256) void k_att_bias(const float* __restrict__ s_hat, int P, int V, int Npad,
                                                   float lambda_max, float eps, float* __restrict__ bias2) {
  const int j = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y;
  if (j >= Npad) return;
  float x = -INFINITY;
  if (j >= P && j < P + V) x = log2f(fmaxf(lambda_max * s_hat[(int64_t)b * V + (j - P)], eps));
  bias2[(int64_t)b * Npad + j] = x;
}

// grid (ceil(Npad/32), Hkv, B), 256 threads; vt[b,g,c,n] = v[b,g,n,c] for n < N, 0 for N <= n < Npad.
// 16-byte loads along d into LDS, 16-byte stores along the keys out of it.
template <typename T>
__global__ __launch_bounds__(256) void k_vtranspose(const T* __restrict__ v, Strides3 sv, int N, int Npad, int d,
                                                     T* __restrict__ vt) {
  constexpr int E = elem<T>::per16;
  __shared__ T tile[32][128 + E];
  const int n0 = blockIdx.x * 32, g = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  const T* src = v + b * sv.b + g * sv.h;
  const int cpr = d / E;                                   // 16-byte chunks per row
  for (int idx = tid; idx < 32 * cpr; idx += 256) {
    const int r = idx / cpr, c = idx - r * cpr;
    uint4 x = make_uint4(0, 0, 0, 0);
    if (n0 + r < N) x = ldg16_stream(src + (int64_t)(n0 + r) * sv.r + c * E);
    *reinterpret_cast<uint4*>(&tile[r][c * E]) = x;
  }
  __syncthreads();
  T* dst = vt + ((int64_t)b * gridDim.y + g) * d * Npad;
  const int gpr = 32 / E;                                  // 16-byte groups of keys per output row
  for (int idx = tid; idx < d * gpr; idx += 256) {
    const int c = idx / gpr, r0 = (idx - c * gpr) * E;
    T x[E];
#pragma unroll
    for (int e = 0; e < E; ++e) x[e] = tile[r0 + e][c];
    uint4 y;
    __builtin_memcpy(&y, x, 16);
    *reinterpret_cast<uint4*>(dst + (int64_t)c * Npad + n0 + r0) = y;
  }
}

__device__ __forceinline__ float fast_exp2_att(float x) { return __builtin_amdgcn_exp2f(x); }

// Floats to the storage type with the hardware's packed conversion (round to nearest even): the
// probabilities are converted once per key tile, which makes the integer version too expensive here.
typedef __bf16 att_bf16x2 __attribute__((ext_vector_type(2)));
typedef float att_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t cvt_pk_bf16(float a, float b) {
  att_f32x2 x = {a, b};
  att_bf16x2 y = __builtin_convertvector(x, att_bf16x2);
  uint32_t u;
  __builtin_memcpy(&u, &y, 4);
  return u;
}
template <typename T> __device__ __forceinline__ uint4 att_pack16(const float* in);
template <> __device__ __forceinline__ uint4 att_pack16<float>(const float* in) { return pack16<float>(in); }
template <> __device__ __forceinline__ uint4 att_pack16<bf16_t>(const float* in) {
  return make_uint4(cvt_pk_bf16(in[0], in[1]), cvt_pk_bf16(in[2], in[3]), cvt_pk_bf16(in[4], in[5]),
                    cvt_pk_bf16(in[6], in[7]));
}

// four consecutive output elements from floats (one rounding to the storage type)
template <typename T> __device__ __forceinline__ void store4(T* dst, const float* f);
template <> __device__ __forceinline__ void store4<float>(float* dst, const float* f) {
  *reinterpret_cast<uint4*>(dst) = pack16<float>(f);
}
template <> __device__ __forceinline__ void store4<bf16_t>(bf16_t* dst, const float* f) {
  *reinterpret_cast<uint2*>(dst) =
      make_uint2(cvt_pk_bf16(f[0], f[1]), cvt_pk_bf16(f[2], f[3]));
}

// key held in accumulator register v of a lane of half hf, relative to the tile
__device__ __forceinline__ int att_key_of(int v, int hf) { return 8 * (v >> 2) + 4 * hf + (v & 3); }

constexpr int ATT_QWG = 256;                   // queries per workgroup

// LDS swizzles: the 16-byte piece p of row r is stored in slot p ^ x(r), so that 16 consecutive rows
// spread over all banks for the strided operand reads while the loads still write 1 KiB at a time
__device__ __forceinline__ int att_kswz(int row, int row_bytes) { return row_bytes <= 128 ? (row >> 1) & 7 : row & 15; }
__device__ __forceinline__ int att_vswz(int row, int row_bytes) { return row_bytes <= 64 ? (row >> 2) & 3 : (row >> 1) & 7; }

// CH = 16-byte chunks of a row per lane half (row bytes = 32 * CH); NW waves of QB 32-query blocks each
template <typename T, int CH, int NW, int QB>
__global__ __launch_bounds__(64 * NW) void k_attention(const T* __restrict__ q, Strides3 sq, const T* __restrict__ k,
                                                    Strides3 sk, const T* __restrict__ vt, int Npad,
                                                    const float* __restrict__ bias2, T* __restrict__ out, int H,
                                                    int Hkv, int N, int P, int V, float c2) {
  constexpr int E = elem<T>::per16;            // elements per 16-byte chunk
  constexpr int D = CH * 2 * E;                // head dimension
  constexpr int DT = D / 32;                   // 32-row tiles of O^T
  constexpr int NPS = 32 / (2 * E);            // contraction steps of the second product per key tile
  constexpr int RB = 32 * CH;                  // bytes of a key row
  constexpr int VB = 32 * (int)sizeof(T);      // bytes of a values^T row per key tile
  constexpr int KTILE = 32 * RB, VTILE = D * VB, STAGE = KTILE + VTILE;
  constexpr int KLD = KTILE / 1024, VLD = VTILE / 1024;     // 1 KiB load instructions per tile
  extern __shared__ __align__(16) char lds[];
  const uint32_t lds_addr = lds_address(lds);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, hf = lane >> 5;
  const int b = blockIdx.z, h = blockIdx.y, g = (h * Hkv) / H;
  const int iw = blockIdx.x * ATT_QWG;          // first query of the workgroup
  constexpr int ATT_QW = 32 * QB;               // queries per wave
  static_assert(NW * ATT_QW == ATT_QWG, "workgroup shape");
  const int i0 = iw + wave * ATT_QW;            // first query of the wave
  const bool bidir = bias2 != nullptr;
  const float inv_c2 = 1.0f / c2;
  const int img_lo = P, img_hi = P + V;         // image span [img_lo, img_hi)

  // keys to visit: up to the last query, or to the end of the image span if image rows are held
  // (their future image keys count, discounted)
  auto last_key = [&](int first, int count) {
    const int hi = min(first + count - 1, N - 1);
    int jl = hi;
    if (bidir && hi >= img_lo && first < img_hi) jl = max(jl, img_hi - 1);
    return first < N ? jl : -1;
  };
  const int jl_wg = last_key(iw, ATT_QWG), jl_w = last_key(i0, ATT_QW);
  const int ntiles = jl_wg / 32 + 1;

  // queries: B operand of S^T, pieces 2c + hf of the row
  uint4 qa[QB][CH];
  int qi[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    qi[qb] = i0 + 32 * qb + n;
    const char* qrow =
        reinterpret_cast<const char*>(q + b * sq.b + h * sq.h + (int64_t)min(qi[qb], N - 1) * sq.r) + hf * 16;
#pragma unroll
    for (int c = 0; c < CH; ++c) qa[qb][c] = ldg16(qrow + c * 32);
  }

  // tile loads: wave w issues the 1 KiB pieces w, w + 4, ... of the key tile and of the values^T tile
  const char* kg = reinterpret_cast<const char*>(k + b * sk.b + g * sk.h);
  const int64_t krow_bytes = sk.r * (int64_t)sizeof(T);
  const char* vg = reinterpret_cast<const char*>(vt + ((int64_t)b * Hkv + g) * D * Npad);
  auto issue_tile = [&](int jt) {
    const uint32_t st = lds_addr + (uint32_t)(jt & 1) * STAGE;
    const int j0 = jt * 32;
#pragma unroll
    for (int u = 0; u < (KLD + NW - 1) / NW; ++u) {
      const int qn = wave + NW * u;
      if (qn < KLD) {
        const int off = qn * 1024 + 16 * lane, row = off / RB, slot = (off % RB) >> 4;
        const int piece = slot ^ att_kswz(row, RB);
        const uint32_t voff = (uint32_t)((int64_t)min(j0 + row, N - 1) * krow_bytes) + piece * 16;
        load_to_lds16(kg, voff, st + qn * 1024);
      }
    }
#pragma unroll
    for (int u = 0; u < (VLD + NW - 1) / NW; ++u) {
      const int qn = wave + NW * u;
      if (qn < VLD) {
        const int off = qn * 1024 + 16 * lane, row = off / VB, slot = (off % VB) >> 4;
        const int piece = slot ^ att_vswz(row, VB);
        const uint32_t voff = (uint32_t)(((int64_t)row * Npad + j0) * sizeof(T)) + piece * 16;
        load_to_lds16(vg, voff, st + KTILE + qn * 1024);
      }
    }
  };

  f32x16_t o[QB][DT];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[qb][t][v] = 0.0f;
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) { m_run[qb] = -INFINITY; l_run[qb] = 0.0f; }

  // operand read offsets inside a tile
  const int k_off = n * RB, k_x = att_kswz(n, RB);
  int v_off[DT], v_x[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t) {
    v_off[t] = (t * 32 + n) * VB;
    v_x[t] = att_vswz(t * 32 + n, VB);
  }

  issue_tile(0);
  wait_all_vmem();
  __syncthreads();
  for (int jt = 0; jt < ntiles; ++jt) {
    if (jt + 1 < ntiles) issue_tile(jt + 1);
    const int j0 = jt * 32;
    if (j0 <= jl_w) {
      const char* Kt = lds + (jt & 1) * STAGE;
      const char* Vt = Kt + KTILE;
      f32x16_t s[QB];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[qb][v] = 0.0f;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const uint4 a = *reinterpret_cast<const uint4*>(Kt + k_off + (((2 * c + hf) ^ k_x) << 4));
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) mma32<T>(s[qb], a, qa[qb][c]);
      }
      uint4 pb[QB][NPS];
      // discounts of this lane's 16 keys (needed only where a key may follow a query)
      float kbias[16];
      const bool masked_tile = j0 + 31 > i0;
      if (masked_tile) {
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          float4 x = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
          if (bidir) x = *reinterpret_cast<const float4*>(bias2 + (int64_t)b * Npad + j0 + 8 * gq + 4 * hf);
          kbias[4 * gq] = x.x; kbias[4 * gq + 1] = x.y; kbias[4 * gq + 2] = x.z; kbias[4 * gq + 3] = x.w;
        }
      }
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const int i = qi[qb];
        float z[16];
        if (j0 + 31 <= i0 + 32 * qb) {           // every key of the tile precedes every query of the block
#pragma unroll
          for (int v = 0; v < 16; ++v) z[v] = s[qb][v];       // raw: the scale goes into the exponent below
        } else if (j0 > i0 + 32 * qb + 31 && i0 + 32 * qb >= img_lo && i0 + 32 * qb + 31 < img_hi) {
          // every key follows every query of the block and all its queries are image rows: the mask
          // is the key's discount (-inf off the image span), whatever the query
#pragma unroll
          for (int v = 0; v < 16; ++v) z[v] = fmaf(kbias[v], inv_c2, s[qb][v]);
        } else {
          const bool q_img = i >= img_lo && i < img_hi;
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int j = j0 + att_key_of(v, hf);
            const float ahead = q_img ? kbias[v] : -INFINITY;      // a key after the query
            z[v] = s[qb][v] + (j <= i ? 0.0f : ahead) * inv_c2;
          }
        }
        float mx = z[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, z[v]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        // maxima are kept in units of the raw products; m_c = c2 * m is what the exponent subtracts
        const float m_new = fmaxf(m_run[qb], mx);   // finite from the first tile on: key 0 precedes every query
        const float alpha = fast_exp2_att((m_run[qb] - m_new) * c2);
        const float m_c = m_new * c2;
        float p[16], psum = 0.0f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          p[v] = fast_exp2_att(fmaf(z[v], c2, -m_c));
          psum += p[v];
        }
        l_run[qb] = l_run[qb] * alpha + psum;
        m_run[qb] = m_new;
        if (__any(alpha != 1.0f)) {              // the running maxima settle after the first tiles
#pragma unroll
          for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[qb][t][v] *= alpha;
        }
#pragma unroll
        for (int c = 0; c < NPS; ++c) pb[qb][c] = att_pack16<T>(&p[c * E]);
      }
#pragma unroll
      for (int c = 0; c < NPS; ++c)
#pragma unroll
        for (int t = 0; t < DT; ++t) {
          uint4 va;
          if (E == 4) {                          // 4 keys of 4 bytes: piece 2c + hf of the row
            va = *reinterpret_cast<const uint4*>(Vt + v_off[t] + (((2 * c + hf) ^ v_x[t]) << 4));
          } else {                               // keys 16c + 4hf + 0..3 and 16c + 8 + 4hf + 0..3: halves of two pieces
            const uint2 lo = *reinterpret_cast<const uint2*>(Vt + v_off[t] + (((2 * c) ^ v_x[t]) << 4) + 8 * hf);
            const uint2 hi = *reinterpret_cast<const uint2*>(Vt + v_off[t] + (((2 * c + 1) ^ v_x[t]) << 4) + 8 * hf);
            va = make_uint4(lo.x, lo.y, hi.x, hi.y);
          }
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) mma32<T>(o[qb][t], va, pb[qb][c]);
        }
    }
    wait_all_vmem();
    __syncthreads();
  }

#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32);
    const float inv = 1.0f / l_tot;
    const int i = qi[qb];
    if (i < N) {
      T* orow = out + (((int64_t)b * H + h) * N + i) * D;
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          float f[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) f[e] = o[qb][t][4 * gq + e] * inv;
          store4<T>(orow + t * 32 + 8 * gq + 4 * hf, f);
        }
    }
  }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
#ifndef ATT_NW
#define ATT_NW 8       /* waves per workgroup: two per SIMD, so that one wave's softmax arithmetic */
#define ATT_QB 1       /* overlaps the other's MFMAs; one 32-query block per wave */
#endif
static int att_npad(const asap_params& p) { return ((p.P + p.V + p.Tmax + 31) / 32) * 32 + 32; }

size_t attention_workspace_bytes(const asap_params& p) {
  const size_t es = p.qk_dtype == ASAP_BF16 ? 2 : 4;
  return align256(es * (size_t)p.B * p.Hkv * p.d * att_npad(p)) + align256(sizeof(float) * (size_t)p.B * att_npad(p));
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
    ASAP_LAUNCH(tm, "k_att_bias", k_att_bias, dim3((Npad + 255) / 256, p.B), dim3(256), 0, st, s_hat, p.P, p.V, Npad,
                p.lambda_max, p.eps, bias2);
  ASAP_LAUNCH(tm, "k_vtranspose", k_vtranspose<T>, dim3(Npad / 32, p.Hkv, p.B), dim3(256), 0, st,
              static_cast<const T*>(v), sv, N, Npad, p.d, vt);
  const float c2 = 1.4426950408889634f / sqrtf((float)p.d);
  const dim3 grid((N + ATT_QWG - 1) / ATT_QWG, p.H, p.B);
  const int ch = p.d / E / 2;
  const size_t lds = 2 * (size_t)(32 * 32 * ch + p.d * 32 * sizeof(T));   // two stages of (K tile + V^T tile)
#define ASAP_ATT(CHV)                                                                                          \
  do {                                                                                                         \
    auto kern = k_attention<T, CHV, ATT_NW, ATT_QB>;                                                                           \
    if (lds > 48 * 1024) {                                                                                     \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                  \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                \
      if (e != hipSuccess) return e;                                                                           \
    }                                                                                                          \
    ASAP_LAUNCH(tm, "k_attention", kern, grid, dim3(64 * ATT_NW), lds, st, static_cast<const T*>(q), sq,               \
                static_cast<const T*>(k), sk, vt, Npad, bidir ? bias2 : nullptr, static_cast<T*>(out), p.H,    \
                p.Hkv, N, p.P, p.V, c2);                                                                       \
  } while (0)
  if (ch == 4) ASAP_ATT(4);
  else if (ch == 8) ASAP_ATT(8);
  else if (ch == 16 && E == 4) {
    if constexpr (E == 4) ASAP_ATT(16);
  } else return hipErrorInvalidValue;
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
