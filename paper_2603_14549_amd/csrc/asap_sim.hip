// Cosine routing of pruned tokens to kept tokens (Sec. 4.2): the one dense contraction of the
// stage, (pruned rows) x (kept rows)^T over the hidden dimension, on the matrix cores, with the
// row arg-max fused into the epilogue.
//
//   k_sim<T, NT>  workgroup tile BM = 128 source rows x BN = 64*NT destination rows.  The hidden
//                 dimension is walked in steps of 128 bytes per row; a step's (BM + BN) x 128 B
//                 panel is staged through LDS (rows padded to 144 B), double buffered, one barrier
//                 per step.  512 threads: 4 consumer waves (2 x 2 over the tile, each 64 x 32*NT =
//                 2 x NT MFMA tiles of 32 x 32) and 4 producer waves that move global -> LDS with
//                 three steps in flight in registers and accumulate the squared norms of the
//                 rows they move (sources once, kept rows every pass).
//                 The grid is one-dimensional and XCD-aware: consecutive workgroup ids go to the 8
//                 XCDs round-robin, so id % 8 picks the XCD and all tiles of one image are given
//                 ids with the same id % 8 -- they then share that XCD's L2 for the kept panel.
#include "asap_device.hpp"
#include "asap_launch.hpp"

namespace asap {

constexpr int SIM_BM = 128;
constexpr int SIM_LDSROW = 144;
constexpr int NUM_XCD = 8;

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// sum of squares of the elements of a 16-byte chunk added to acc
template <typename T> __device__ __forceinline__ float sumsq16(const uint4& c, float acc);
template <> __device__ __forceinline__ float sumsq16<bf16_t>(const uint4& c, float acc) {
  bf16x2_t p;
  __builtin_memcpy(&p, &c.x, 4); acc = __builtin_amdgcn_fdot2_f32_bf16(p, p, acc, false);
  __builtin_memcpy(&p, &c.y, 4); acc = __builtin_amdgcn_fdot2_f32_bf16(p, p, acc, false);
  __builtin_memcpy(&p, &c.z, 4); acc = __builtin_amdgcn_fdot2_f32_bf16(p, p, acc, false);
  __builtin_memcpy(&p, &c.w, 4); acc = __builtin_amdgcn_fdot2_f32_bf16(p, p, acc, false);
  return acc;
}
template <> __device__ __forceinline__ float sumsq16<float>(const uint4& c, float acc) {
  float f[4];
  unpack16<float>(c, f);
  acc = fmaf(f[0], f[0], acc); acc = fmaf(f[1], f[1], acc);
  acc = fmaf(f[2], f[2], acc); acc = fmaf(f[3], f[3], acc);
  return acc;
}

// k_sim: 512 threads = 4 consumer waves (MFMA, 2 x 2 over the tile) + 4 producer waves (global -> LDS).
// A producer thread moves the 16-byte piece t % 8 of rows t / 8 + 32 i of every step's panel; it keeps
// three steps in registers (issued at step s for step s + 3, written to LDS at step s + 2), so that
// HBM latency is covered by two steps of MFMA work, and it accumulates the squared norms of its
// source rows.  Consumers only read LDS and issue MFMAs.  Both roles meet at one barrier per step.
template <typename T, int NT>
__global__ __launch_bounds__(512) void k_sim(const T* __restrict__ xv, int64_t sb, int64_t sr, int D,
                                              const int32_t* __restrict__ pruned, const int32_t* __restrict__ kept,
                                              int B, int M, int k, int mtiles,
                                              float threshold, int32_t* __restrict__ assign,
                                              float* __restrict__ best_sim) {
  constexpr int BN = 64 * NT;
  constexpr int ROWS = SIM_BM + BN;
  constexpr int PP = ROWS / 32;                  // 16-byte pieces a producer thread moves per step
  constexpr int PA = SIM_BM / 32;                // of which source rows
  constexpr int STAGE = ROWS * SIM_LDSROW;
  extern __shared__ __align__(16) char lds[];
  float* norm2 = reinterpret_cast<float*>(lds + 2 * STAGE);   // [BM]
  float* part_v = norm2 + SIM_BM;                             // [2][BM]
  int* part_c = reinterpret_cast<int*>(part_v + 2 * SIM_BM);  // [2][BM]
  float* normk = reinterpret_cast<float*>(part_c + 2 * SIM_BM);  // [BN] squared norms of this pass's kept rows

  // XCD-aware decode of the linear workgroup id
  const int xcd = blockIdx.x % NUM_XCD, slot = blockIdx.x / NUM_XCD;
  const int b = (slot / mtiles) * NUM_XCD + xcd;
  if (b >= B) return;
  const int m0 = (slot % mtiles) * SIM_BM;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool producer = wave >= 4;
  const int n = lane & 31, hf = lane >> 5;
  const int wm = (wave >> 1) & 1, wn = wave & 1;
  const int ltid = tid & 255, piece = ltid & 7, rbase = ltid >> 3;
  const char* xb = reinterpret_cast<const char*>(xv + b * sb);
  const int64_t rowb = sr * (int64_t)sizeof(T);
  const int steps = (D * (int)sizeof(T)) / 128;
  const int npass = (k + BN - 1) / BN;
  // Every workgroup walks the hidden dimension from its own starting step: rows are a power-of-two
  // number of bytes apart, so workgroups in lockstep would all hit the same memory channel.
  const int rot = ((slot % mtiles) + 16 * (slot / mtiles)) % steps;

  float run_v = -INFINITY;   // running best over destination passes (consumer threads < BM)
  int run_c = 0;

  if (producer) {
    // byte offsets of this thread's rows from the image base (an image spans < 4 GiB)
    uint32_t off[PP];
#pragma unroll
    for (int i = 0; i < PA; ++i) {
      int r = min(m0 + rbase + 32 * i, M - 1);
      off[i] = (uint32_t)(pruned[(int64_t)b * M + r] * rowb + piece * 16);
    }
    float ss[PP];
#pragma unroll
    for (int i = 0; i < PP; ++i) ss[i] = 0.0f;
    for (int pass = 0; pass < npass; ++pass) {
      const bool count_src = pass == 0;
#pragma unroll
      for (int i = PA; i < PP; ++i) {
        int c = min(pass * BN + rbase + 32 * (i - PA), k - 1);
        off[i] = (uint32_t)(kept[(int64_t)b * k + c] * rowb + piece * 16);
        ss[i] = 0.0f;
      }
      uint4 st[3][PP];
      auto fetch = [&](uint4 (&dst)[PP], int s) {
        int sr_ = s + rot; if (sr_ >= steps) sr_ -= steps;   // rotated walk, see rot
        const char* base = xb + (int64_t)sr_ * 128;
#pragma unroll
        for (int i = 0; i < PP; ++i) dst[i] = ldg16(base + off[i]);
      };
      auto stash = [&](const uint4 (&src)[PP], int buf) {
        char* dst = lds + buf * STAGE + rbase * SIM_LDSROW + piece * 16;
#pragma unroll
        for (int i = 0; i < PP; ++i) {
          *reinterpret_cast<uint4*>(dst + i * 32 * SIM_LDSROW) = src[i];
          if (i >= PA || count_src) ss[i] = sumsq16<T>(src[i], ss[i]);
        }
      };
      // step s with R = s % 3: the set of step s + 1 goes to LDS, set R is refilled for step s + 3
      auto pstep = [&](int s, auto r) {
        constexpr int R = decltype(r)::value;
        if (wave & 1) {       // half of the producer waves load first, so LDS writes and global loads overlap
          if (s + 3 < steps) fetch(st[R], s + 3);
          if (s + 1 < steps) stash(st[(R + 1) % 3], (s + 1) & 1);
        } else {
          if (s + 1 < steps) stash(st[(R + 1) % 3], (s + 1) & 1);
          if (s + 3 < steps) fetch(st[R], s + 3);
        }
        __syncthreads();
      };
      fetch(st[0], 0);
      if (steps > 1) fetch(st[1], 1);
      if (steps > 2) fetch(st[2], 2);
      stash(st[0], 0);
      __syncthreads();
      for (int s = 0; s < steps;) {
        pstep(s, std::integral_constant<int, 0>{});
        if (++s >= steps) break;
        pstep(s, std::integral_constant<int, 1>{});
        if (++s >= steps) break;
        pstep(s, std::integral_constant<int, 2>{});
        ++s;
      }
      // squared norms of the rows this thread moved: 8 consecutive lanes share a row
#pragma unroll
      for (int i = 0; i < PP; ++i) {
        float v = ss[i];
        v += __shfl_xor(v, 1);
        v += __shfl_xor(v, 2);
        v += __shfl_xor(v, 4);
        if (piece == 0) {
          if (i >= PA) normk[rbase + 32 * (i - PA)] = v;
          else if (count_src) norm2[rbase + 32 * i] = v;
        }
      }
      __syncthreads();   // norms visible to the consumers' epilogue
      __syncthreads();
      __syncthreads();
    }
  } else {
    for (int pass = 0; pass < npass; ++pass) {
      const int n0 = pass * BN;
      f32x16_t acc[2][NT];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[i][t][v] = 0.0f;
      __syncthreads();
      for (int s = 0; s < steps; ++s) {
        // LDS operand reads run one contraction slice ahead of the MFMAs that use them
        const char* A = lds + (s & 1) * STAGE + (wm * 64 + n) * SIM_LDSROW + hf * 64;
        const char* Bp = lds + (s & 1) * STAGE + (SIM_BM + wn * (BN / 2) + n) * SIM_LDSROW + hf * 64;
        uint4 a[2][2], bq[2][NT];
        auto load_ops = [&](int set, int kk) {
          a[set][0] = *reinterpret_cast<const uint4*>(A + kk * 16);
          a[set][1] = *reinterpret_cast<const uint4*>(A + 32 * SIM_LDSROW + kk * 16);
#pragma unroll
          for (int t = 0; t < NT; ++t)
            bq[set][t] = *reinterpret_cast<const uint4*>(Bp + t * 32 * SIM_LDSROW + kk * 16);
        };
        load_ops(0, 0);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          if (kk < 3) load_ops((kk + 1) & 1, kk + 1);
          __builtin_amdgcn_sched_barrier(0);     // keep the next slice's reads ahead of this slice's MFMAs
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            mma32<T>(acc[0][t], a[kk & 1][0], bq[kk & 1][t]);
            mma32<T>(acc[1][t], a[kk & 1][1], bq[kk & 1][t]);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
      }
      // row arg-max of dot / |x_i| over this pass's destinations (|x_j| > 0 does not move it)
      __syncthreads();   // the producers' norms
      float invk[NT];
      int colv[NT];
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int cl = wn * (BN / 2) + t * 32 + n;
        colv[t] = n0 + cl;
        invk[t] = colv[t] < k ? 1.0f / fmaxf(sqrtf(normk[cl]), 1e-8f) : 0.0f;
      }
      // Each lane first takes the best of its NT columns per row; the 32 lanes that share a row then
      // exchange through LDS (the stage buffers are idle now): one lane per row scans the 32 partial
      // results.  Lanes of one wave only talk to each other here, and a wave's LDS operations are
      // carried out in order, so no barrier is needed.
      {
        constexpr int PITCH = 32 * 8 + 8;
        char* scr = lds + wave * (32 * PITCH);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            float bv = -INFINITY;
            int bc = 0x7fffffff;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
              float c = acc[i][t][v] * invk[t];
              bool take = (colv[t] < k) & (c > bv);      // columns ascend with t: strict > keeps the smaller
              bv = take ? c : bv;
              bc = take ? colv[t] : bc;
            }
            *reinterpret_cast<uint2*>(scr + mma32_row(v, lane) * PITCH + n * 8) =
                make_uint2(__float_as_uint(bv), (uint32_t)bc);
          }
          if (lane < 32) {
            float bv = -INFINITY;
            int bc = 0x7fffffff;
#pragma unroll
            for (int e = 0; e < 32; ++e) {
              uint2 u = *reinterpret_cast<const uint2*>(scr + lane * PITCH + e * 8);
              float ov = __uint_as_float(u.x);
              int oc = (int)u.y;
              bool take = (ov > bv) | ((ov == bv) & (oc < bc));
              bv = take ? ov : bv;
              bc = take ? oc : bc;
            }
            int row = wm * 64 + i * 32 + lane;
            part_v[wn * SIM_BM + row] = bv;
            part_c[wn * SIM_BM + row] = bc;
          }
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
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
size_t sim_workspace_bytes(const asap_params&) { return 0; }

template <typename T, int NT>
static hipError_t launch_sim_nt(const asap_params& p, const T* xv, int64_t sb, int64_t sr, const int32_t* pruned,
                                const int32_t* kept, int32_t* assign, float* best_sim,
                                hipStream_t st, Timer* tm) {
  constexpr int BN = 64 * NT, ROWS = SIM_BM + BN;
  const size_t lds = 2 * (size_t)ROWS * SIM_LDSROW + sizeof(float) * (5 * SIM_BM + BN);
  auto kern = k_sim<T, NT>;
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  const int M = p.V - p.k;
  const int mtiles = (M + SIM_BM - 1) / SIM_BM;
  const int groups = (p.B + NUM_XCD - 1) / NUM_XCD;
  ASAP_LAUNCH(tm, "k_sim", kern, dim3(NUM_XCD * groups * mtiles), dim3(512), lds, st, xv, sb, sr, p.D, pruned,
              kept, p.B, M, p.k, mtiles, p.sim_threshold, assign, best_sim);
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
static hipError_t sim_typed(const asap_params& p, const void* hidden, int64_t hsb, int64_t hsr,
                            const int32_t* kept, const int32_t* pruned, int32_t* assign, float* best_sim,
                            char* ws, hipStream_t st, Timer* tm) {
  const T* xv = static_cast<const T*>(hidden) + (int64_t)p.P * hsr;
  (void)ws;
  switch (pick_nt(p.k)) {
    case 1: return launch_sim_nt<T, 1>(p, xv, hsb, hsr, pruned, kept, assign, best_sim, st, tm);
    case 2: return launch_sim_nt<T, 2>(p, xv, hsb, hsr, pruned, kept, assign, best_sim, st, tm);
    case 3: return launch_sim_nt<T, 3>(p, xv, hsb, hsr, pruned, kept, assign, best_sim, st, tm);
    case 4: return launch_sim_nt<T, 4>(p, xv, hsb, hsr, pruned, kept, assign, best_sim, st, tm);
    default: return launch_sim_nt<T, 5>(p, xv, hsb, hsr, pruned, kept, assign, best_sim, st, tm);
  }
}

hipError_t launch_similarity(const asap_params& p, const void* hidden, int64_t hsb, int64_t hsr,
                             const int32_t* kept, const int32_t* pruned, int32_t* assign, float* best_sim,
                             char* ws, hipStream_t st, Timer* tm) {
  if (p.h_dtype == ASAP_BF16)
    return sim_typed<bf16_t>(p, hidden, hsb, hsr, kept, pruned, assign, best_sim, ws, st, tm);
  return sim_typed<float>(p, hidden, hsb, hsr, kept, pruned, assign, best_sim, ws, st, tm);
}

}  // namespace asap
