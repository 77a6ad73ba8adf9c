// asap_score: Eq. 2 (raw attention mass), Eq. 3 (salience), Eq. 4 (discount) and the text-row
// softmax of Eq. 5 reduced to one selection score per visual token.
//
// Kernels, in launch order:
//   k_qsum        column sums of the visual queries per (image, head[, row chunk]); rows are added
//                 eight at a time in fp32, the eights in fp64
//   k_qsplit      fixed-order sum of those partials per kv head (fp64), also split into four bf16
//                 pieces per component (32 significant bits) for the matrix cores
//   k_mass_mfma   s_j = sum_g qbar_g . k_{g,j} / (H sqrt d)  (Eq. 2 by linearity) and the per-image
//                 min / max of s through order-preserving integer atomics.  The four pieces of
//                 qbar are four query rows of an MFMA tile; bf16 keys enter as they are, f32 keys
//                 as three bf16 pieces each (hi + mid + lo = the key to 2^-27), so every product is
//                 exact; one head's 128 products per piece pair are added in fp32 by the matrix
//                 instruction, everything above that in fp64.
//                 When the text rows that rank the tokens are few (rows of a kv head's query heads
//                 <= 28, bf16), they ride in the free rows of that tile: the sweep then also leaves
//                 their raw logits in the workspace, and no further sweep over the keys is needed.
//                 Small batches cut the kv heads into groups with workgroups of their own, which
//                 leave partial masses; k_mass_finish adds them and takes min / max.
//   either the two sweeps over the keys
//   k_attn_stats  per (image, head, key split): key x text-query logits on the matrix cores (keys as
//                 tile rows, so a lane owns one text row), online (max, sum) of lambda'_j 2^z per row
//   k_attn_colsum the sweep again with queries as tile rows and the merged row statistics:
//                 normalised column sums per key
//   or, from stored logits,
//   k_rowstats_logits / k_colsum_logits   the same two reductions over the [rows, V] logits
//   k_score       fixed-order head reduction, times lambda' (Eq. 4) in fp64, mean over heads and
//                 text rows; also writes s_hat (Eq. 3)
//   k_score_select  the same followed by the top-k selection of asap_select in one launch (one
//                 workgroup per image), when the stage runs as one call; k_score_select_kv has further
//                 workgroups that copy the K/V rows of prefix and text meanwhile
// f32 queries and keys reach the bf16 matrix instructions as three bf16 pieces each; a logit is the
// sum of the six piece products that matter (hi.hi, hi.mid, mid.hi, mid.mid, hi.lo, lo.hi: what is
// left out is below 2^-25 of sum |q_c k_c|, half a unit of the fp32 accumulation itself).
// Logits stay in accumulator units; the factor log2(e)/sqrt(d) is applied to differences from the
// row maximum only, so its rounding error scales with the distance from the maximum.
#include "asap_device.hpp"
#include "asap_launch.hpp"
#include "asap_select.hpp"

namespace asap {

// order-preserving map double <-> uint64 (for atomic min / max)
__device__ __forceinline__ unsigned long long f64_key(double x) {
  unsigned long long u = (unsigned long long)__double_as_longlong(x);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}
__device__ __forceinline__ double f64_unkey(unsigned long long k) {
  unsigned long long u = (k >> 63) ? (k & 0x7fffffffffffffffull) : ~k;
  return __longlong_as_double((long long)u);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// successive bf16 roundings of what is left of x: x = p0 + p1 + p2 + p3 to 32 significant bits
__device__ __forceinline__ void split_bf16x4(double x, uint16_t* out, int stride) {
  double rest = x;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    uint32_t bits = f32_to_bf16_bits((float)rest);
    out[p * stride] = (uint16_t)bits;
    rest -= (double)bf16_bits_to_f32(bits);
  }
}

// ------------------------------------------------------------------------------------------
// k_qsum: grid (chunks, H, B), 1024 threads.  A row is d elements = LPR 16-byte pieces; thread t
// keeps piece t % LPR of rows t / LPR + RPI * i.  Block (0, 0, b) also resets the min / max keys.
// With one chunk and one query head per kv head the block's sums are final (`direct`): it writes
// qbar and its bf16 split itself and k_qsplit is not needed.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(1024) void k_qsum(const T* __restrict__ q, Strides3 sq, int V, int d, int R,
                                                double* __restrict__ qpart, unsigned long long* __restrict__ mmkey,
                                                double* __restrict__ qbar, uint16_t* __restrict__ qsplit, int direct) {
  constexpr int E = elem<T>::per16;
  const int LPR = d / E, RPI = 1024 / LPR;
  const int tid = threadIdx.x, piece = tid % LPR, r0 = tid / LPR;
  const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (c == 0 && h == 0 && tid == 0) { mmkey[2 * b] = ~0ull; mmkey[2 * b + 1] = 0ull; }
  const int lo = c * R, hi = min(V, lo + R);
  const char* base = reinterpret_cast<const char*>(q + b * sq.b + h * sq.h + piece * E);
  const int64_t rowb = sq.r * (int64_t)sizeof(T);
  double acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.0;
  int row = lo + r0;
  for (; row + 7 * RPI < hi; row += 8 * RPI) {       // eight rows in flight, summed in fp32
    uint4 ch[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) ch[u] = ldg16_stream(base + (int64_t)(row + u * RPI) * rowb);
    float f[E], g[E];
    unpack16<T>(ch[0], f);
#pragma unroll
    for (int u = 1; u < 8; ++u) {
      unpack16<T>(ch[u], g);
#pragma unroll
      for (int e = 0; e < E; ++e) f[e] += g[e];
    }
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] += (double)f[e];
  }
  for (; row < hi; row += RPI) {
    float f[E];
    unpack16<T>(ldg16(base + (int64_t)row * rowb), f);
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] += (double)f[e];
  }
  // fixed-order reduction: row groups inside a wave by butterfly, then the 16 waves through LDS
  __shared__ double red[16 * 128];
  const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    double a = acc[e];
    for (int off = LPR; off < 64; off <<= 1) a += shfl_xor_f64(a, off);
    if (lane < LPR) red[wave * d + piece * E + e] = a;
  }
  __syncthreads();
  if (tid < d) {
    double s = 0.0;
    for (int w = 0; w < 16; ++w) s += red[w * d + tid];
    qpart[(((int64_t)b * gridDim.y + h) * gridDim.x + c) * d + tid] = s;
    if (direct) {
      qbar[((int64_t)b * gridDim.y + h) * d + tid] = s;
      split_bf16x4(s, qsplit + ((int64_t)b * gridDim.y + h) * 4 * d + tid, d);
    }
  }
}

// k_qsplit: grid (Hkv, B), d threads.  qbar[b,g,:] = sum over the heads of group g and the chunks;
// qsplit[b,g,p,:] (p = 0..3) = successive bf16 roundings of what is left of qbar.
__global__ void k_qsplit(const double* __restrict__ qpart, double* __restrict__ qbar, uint16_t* __restrict__ qsplit,
                         int H, int Hkv, int nchunk, int d, unsigned long long* __restrict__ mmkey) {
  const int g = blockIdx.x, b = blockIdx.y, c = threadIdx.x;
  const int G = H / Hkv;
  if (g == 0 && c == 0) { mmkey[2 * b] = ~0ull; mmkey[2 * b + 1] = 0ull; }   // also where k_qsum did not run
  // the partials of the group's heads and chunks lie one after the other (head-major): added in that
  // order, eight loads in flight
  const double* src = qpart + ((int64_t)b * H + g * G) * nchunk * d + c;
  const int n = G * nchunk;
  double s = 0.0;
  for (int i0 = 0; i0 < n; i0 += 8) {
    double part[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) part[u] = i0 + u < n ? src[(int64_t)(i0 + u) * d] : 0.0;
#pragma unroll
    for (int u = 0; u < 8; ++u) s += part[u];
  }
  qbar[((int64_t)b * Hkv + g) * d + c] = s;
  split_bf16x4(s, qsplit + ((int64_t)b * Hkv + g) * 4 * d + c, d);
}

__device__ __forceinline__ void publish_minmax(unsigned long long kmin, unsigned long long kmax, bool active,
                                               unsigned long long* blk_mm, unsigned long long* mmkey, int b) {
  if (active) {
    atomicMin(&blk_mm[0], kmin);
    atomicMax(&blk_mm[1], kmax);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    atomicMin(&mmkey[2 * b], blk_mm[0]);
    atomicMax(&mmkey[2 * b + 1], blk_mm[1]);
  }
}

// A lane's share of one contraction group (8 elements): one 16-byte chunk of bf16, two of f32.
template <typename T> struct group_bytes;
template <> struct group_bytes<bf16_t> { static constexpr int value = 16; };
template <> struct group_bytes<float> { static constexpr int value = 32; };

// Text rows that ride in the mass sweep (bf16 only).  Rows 4 .. 4 + R - 1 of the A tile of kv head g
// hold text row t = r % T_eff of query head g G + r / T_eff; their logits against every key go to
// zlog [B, H, T_eff, V].
struct RideArgs {
  const void* qt; Strides3 sq;      // [B,H,Tmax,d]
  const int32_t* text_len;          // [B]
  float* zlog;
  int H, G, T_eff, Tmax, last_only;
};

// ------------------------------------------------------------------------------------------
// k_mass_mfma: grid (ceil(V/32), B * HS), 256 threads = 4 waves.  A workgroup owns one 32-key tile
// and the kv heads of group hs (Hkv / HS of them); wave w walks the heads g_lo + w, g_lo + w + 4, ...
// The four bf16 pieces of qbar_g are rows 0..3 of the MFMA A tile (rows 4..31 are zero, or text
// rows that ride along), the keys are the B tile, so lane n (< 32) finds the four partial dot
// products of key n in its first four accumulator registers.
// The tile of a head is an isolated piece of memory (8 KiB for bf16, d = 128), and reading such
// pieces in the operand pattern (32 rows x 32 bytes per instruction) was measured at 4.2 TB/s against
// 6.0 TB/s for whole rows.  So a wave reads whole rows (LPR consecutive lanes per row) and turns the
// tile into the operand layout through an LDS buffer of its own -- written and read by the same
// wave, in order, so no barrier is involved.  NG = contraction groups of 8 elements (d = 16 NG).
// HS == 1: writes s64, s_raw and publishes min / max; HS > 1: writes the group's partial mass to
// spart [HS, B, V] for k_mass_finish.
// ------------------------------------------------------------------------------------------
template <typename T, int NG, bool RIDE>
__global__ __launch_bounds__(256, (sizeof(T) == 4 ? 2 : RIDE ? 3 : 1)) void k_mass_mfma(const T* __restrict__ kv, Strides3 sk,
                                                    const uint16_t* __restrict__ qsplit, int Hkv, int V, int HS,
                                                    double scale, double* __restrict__ s64, float* __restrict__ s_raw,
                                                    unsigned long long* __restrict__ mmkey,
                                                    double* __restrict__ spart, RideArgs ra) {
  constexpr int GB = group_bytes<T>::value;
  constexpr int RBY = NG * 2 * GB;                    // row bytes
  constexpr int LPR = RBY / 16, RPI = 64 / LPR;       // lanes per row, rows per load instruction
  constexpr int NL = 32 / RPI;                        // load instructions per tile
  constexpr int NC = GB / 16;                         // 16-byte chunks per group and lane
  constexpr bool F32 = GB == 32;
  static_assert(!RIDE || !F32, "text rows ride with bf16 keys only");
  // one register set for the key rows (reloaded as soon as it is staged) where a second would cost a
  // workgroup per compute unit: f32 rows, and the kernel that also carries text rows
  constexpr bool REUSE = F32 || RIDE;
  __shared__ __align__(16) char stage[4][32 * RBY];
  __shared__ double part[4][32];
  __shared__ unsigned long long blk_mm[2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, hf = lane >> 5;
  const int piece = lane % LPR, r0 = lane / LPR;
  const int b = blockIdx.y / HS, hs = blockIdx.y % HS, j0 = blockIdx.x * 32;
  const int g_lo = hs * (Hkv / HS), g_hi = g_lo + Hkv / HS;
  if (tid == 0) { blk_mm[0] = ~0ull; blk_mm[1] = 0ull; }
  const int64_t headb = sk.h * (int64_t)sizeof(T);
  // LDS: the 16-byte piece p of row r sits in slot p ^ x(r): whole-row writes and operand reads of 16
  // consecutive rows both cover all banks
  auto swz = [](int row) { return LPR == 8 ? (row >> 1) & 7 : row & (LPR - 1); };
  char* st = stage[wave];
  uint32_t roff[NL];          // byte offsets inside one head of one image (< 2 GiB, checked on the host)
  int wr[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int row = r0 + RPI * i;
    roff[i] = (uint32_t)(min(j0 + row, V - 1) * (int)sk.r * (int)sizeof(T) + piece * 16);
    wr[i] = row * RBY + ((piece ^ swz(row)) << 4);
  }
  // operand read (c, u): piece NC (2c + hf) + u of row n
  int rd[NG][NC];
#pragma unroll
  for (int c = 0; c < NG; ++c)
#pragma unroll
    for (int u = 0; u < NC; ++u) rd[c][u] = n * RBY + (((NC * (2 * c + hf) + u) ^ swz(n)) << 4);
  const char* kbase = reinterpret_cast<const char*>(kv + b * sk.b);
  // lane (m, hf) with m < 4 supplies piece m of qbar_g, half hf of each group's components
  const char* qbase = reinterpret_cast<const char*>(qsplit + ((int64_t)b * Hkv * 4 + (n & 3)) * (NG * 16)) + hf * 16;
  const int64_t qheadb = (int64_t)4 * NG * 16 * 2;
  // text rows that ride: lane n in [4, 4 + R) supplies text row (n - 4) % T_eff of query head g G + (n - 4) / T_eff
  int ride_rows = 0, ride_head = 0;
  const char* tbase = nullptr;
  bool ride_src = false;
  if (RIDE) {
    ride_rows = ra.G * ra.T_eff;
    const int r = n - 4;
    if (r >= 0 && r < ride_rows) {
      const int len = min(max(ra.text_len[b], 0), ra.Tmax);
      const int t = r % ra.T_eff;
      ride_head = r / ra.T_eff;
      const int src = ra.last_only ? len - 1 : t;
      ride_src = ra.last_only ? len >= 1 : t < len;         // padding rows stay zero operands
      tbase = reinterpret_cast<const char*>(static_cast<const bf16_t*>(ra.qt) + b * ra.sq.b +
                                            (int64_t)max(src, 0) * ra.sq.r) + hf * 16;
    }
  }
  const int64_t theadb = RIDE ? ra.sq.h * 2 : 0;
  const bool has_q = n < 4;
  auto load_a = [&](uint4 (&qa)[NG], int g) {
    if (has_q) {
#pragma unroll
      for (int c = 0; c < NG; ++c) qa[c] = ldg16(qbase + g * qheadb + c * 32);
    } else if (RIDE && ride_src) {
      const char* tp = tbase + (int64_t)(g * ra.G + ride_head) * theadb;
#pragma unroll
      for (int c = 0; c < NG; ++c) qa[c] = ldg16(tp + c * 32);
    }
  };
  uint4 qa[NG], kb[NL], kn[NL];
#pragma unroll
  for (int c = 0; c < NG; ++c) qa[c] = make_uint4(0, 0, 0, 0);
  int g = g_lo + wave;
  if (g < g_hi) {
#pragma unroll
    for (int i = 0; i < NL; ++i) kb[i] = ldg16(kbase + g * headb + roff[i]);
    load_a(qa, g);
  }
  double sum = 0.0;
  for (; g < g_hi; g += 4) {
    const int gn = g + 4;
    if (!REUSE && gn < g_hi) {
#pragma unroll
      for (int i = 0; i < NL; ++i) kn[i] = ldg16(kbase + gn * headb + roff[i]);
    }
#pragma unroll
    for (int i = 0; i < NL; ++i) *reinterpret_cast<uint4*>(st + wr[i]) = kb[i];
    if (REUSE && gn < g_hi) {    // the next head's rows reuse this head's registers once those are staged
#pragma unroll
      for (int i = 0; i < NL; ++i) kb[i] = ldg16(kbase + gn * headb + roff[i]);
    }
    if constexpr (!F32) {
      f32x16_t acc;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
      for (int c = 0; c < NG; ++c) mma32<bf16_t>(acc, qa[c], *reinterpret_cast<const uint4*>(st + rd[c][0]));
      sum += ((double)acc[0] + (double)acc[1]) + ((double)acc[2] + (double)acc[3]);   // rows 0..3 (lanes < 32)
      if (RIDE) {
        // wave-uniform base + 32-bit lane offset: row r of this head group's [G T_eff, V] block, key j0 + n
        float* zl = ra.zlog + ((int64_t)(b * ra.H + g * ra.G) * ra.T_eff) * V;
        const uint32_t lane_off = (uint32_t)((4 * hf - 4) * V + j0 + n);      // wraps for hf = 0; the sums below do not
        if (j0 + n < V) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int r = 8 * (v >> 2) + 4 * hf + (v & 3) - 4;
            if (r >= 0 && r < ride_rows) zl[lane_off + (uint32_t)((8 * (v >> 2) + (v & 3)) * V)] = acc[v];
          }
        }
      }
    } else {
      // key pieces as three B tiles; the accumulators of the three are added in fp64
      f32x16_t ah, am, al;
#pragma unroll
      for (int v = 0; v < 16; ++v) { ah[v] = 0.0f; am[v] = 0.0f; al[v] = 0.0f; }
#pragma unroll
      for (int c = 0; c < NG; ++c) {
        const Split3 k3 = split_f32x8(*reinterpret_cast<const uint4*>(st + rd[c][0]),
                                      *reinterpret_cast<const uint4*>(st + rd[c][NC - 1]));
        mma32<bf16_t>(al, qa[c], k3.lo);
        mma32<bf16_t>(am, qa[c], k3.mid);
        mma32<bf16_t>(ah, qa[c], k3.hi);
      }
      const double l = ((double)al[0] + (double)al[1]) + ((double)al[2] + (double)al[3]);
      const double m = ((double)am[0] + (double)am[1]) + ((double)am[2] + (double)am[3]);
      const double h = ((double)ah[0] + (double)ah[1]) + ((double)ah[2] + (double)ah[3]);
      sum += (l + m) + h;
    }
    if (gn < g_hi) {
      load_a(qa, gn);      // small, cached: not worth registers of its own
      if (!REUSE) {
#pragma unroll
        for (int i = 0; i < NL; ++i) kb[i] = kn[i];
      }
    }
  }
  if (hf == 0) part[wave][n] = sum;
  __syncthreads();
  unsigned long long kmin = ~0ull, kmax = 0ull;
  const int j = j0 + n;
  if (tid < 32 && j < V) {
    const double tot = ((part[0][n] + part[1][n]) + part[2][n]) + part[3][n];
    if (HS == 1) {
      const double s = tot * scale;
      s64[(int64_t)b * V + j] = s;
      s_raw[(int64_t)b * V + j] = (float)s;
      kmin = kmax = f64_key(s);
    } else {
      spart[((int64_t)hs * gridDim.y / HS + b) * V + j] = tot;
    }
  }
  if (HS == 1) publish_minmax(kmin, kmax, tid < 32, blk_mm, mmkey, b);
}

// k_mass_finish: grid (B), 1024 threads: adds the HS partial masses of every key in group order,
// scales, writes s64 / s_raw and the image's min / max keys.
__global__ __launch_bounds__(1024) void k_mass_finish(const double* __restrict__ spart, int HS, int B, int V,
                                                       double scale, double* __restrict__ s64,
                                                       float* __restrict__ s_raw,
                                                       unsigned long long* __restrict__ mmkey) {
  __shared__ unsigned long long blk_mm[2];
  const int b = blockIdx.x, tid = threadIdx.x;
  if (tid == 0) { blk_mm[0] = ~0ull; blk_mm[1] = 0ull; }
  __syncthreads();
  unsigned long long kmin = ~0ull, kmax = 0ull;
  for (int j = tid; j < V; j += 1024) {
    double t = 0.0;
    for (int q0 = 0; q0 < HS; q0 += 8) {       // eight loads in flight, added in group order
      double part[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) part[u] = q0 + u < HS ? spart[((int64_t)(q0 + u) * B + b) * V + j] : 0.0;
#pragma unroll
      for (int u = 0; u < 8; ++u) t += part[u];
    }
    const double s = t * scale;
    s64[(int64_t)b * V + j] = s;
    s_raw[(int64_t)b * V + j] = (float)s;
    const unsigned long long key = f64_key(s);
    kmin = key < kmin ? key : kmin;
    kmax = key > kmax ? key : kmax;
  }
  // wave first (1024 same-address LDS atomics would take longer than everything else here)
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const unsigned long long omin = __shfl_xor(kmin, off), omax = __shfl_xor(kmax, off);
    kmin = omin < kmin ? omin : kmin;
    kmax = omax > kmax ? omax : kmax;
  }
  if ((tid & 63) == 0) {
    atomicMin(&blk_mm[0], kmin);
    atomicMax(&blk_mm[1], kmax);
  }
  __syncthreads();
  if (tid == 0) { mmkey[2 * b] = blk_mm[0]; mmkey[2 * b + 1] = blk_mm[1]; }
}

// ------------------------------------------------------------------------------------------
// Text-row attention sweeps.  grid (H * RP * S, B), 256 threads = 4 waves; blockIdx.x = h + H (rp + RP sp).
//   A workgroup takes one (image, head), one pair rp of 32-row blocks of text queries (64 rows; RP
//   pairs cover Tmax) and one key-range split sp.  Two row blocks per workgroup keep its registers and
//   LDS small enough for two workgroups per compute unit, whose waves fill each other's gaps (one
//   wave's exponentials and operand splitting under the other's matrix instructions); longer text
//   costs another workgroup per 64 rows, which reads the keys again -- the pairs of one head are
//   32 ids apart in the launch order, so they run close in time on the same XCD and the second finds
//   the keys in its L2 -- and an image whose own text ends before a pair starts pays nothing for it
//   (the workgroup leaves at once).  The body is compiled for one and for two row blocks and picked by
//   the image's own text length.
//   NG = contraction groups of 8 elements (d = 16 NG).  bf16 queries stay in registers as MFMA
//   operands; f32 queries are split into bf16 pieces once and read from LDS.
// Every wave streams its own 32-key tiles of the split's key range straight from global memory:
// lane (n, hf) of a tile reads, for group c, the bytes [GB (2c + hf), + GB) of key n (GB = 16 for
// bf16, 32 for f32) -- the two lanes of a key take contiguous bytes, which halves the cache lines a
// load instruction touches -- and the query side holds the same elements of its row.
// ------------------------------------------------------------------------------------------
struct AttnArgs {
  const void* qt; Strides3 sq;          // [B,H,Tmax,d]
  const void* kv; Strides3 sk;          // [B,Hkv,V,d]
  const double* s64;                    // [B,V]
  const unsigned long long* mmkey;      // [B,2]
  const int32_t* text_len;              // [B]
  const float* lse_extra;               // [B,H,Tmax] or null
  float* pstat;                         // [B,H,S,2,NR]   partial (max, sum) per text row, NR = 64 RP
  float* upart;                         // [B,H,RP,V]     column sums per head and row pair
  float* zlog;                          // [B,H,T_eff,V]  stored logits (k_rowstats_logits / k_colsum_logits / k_colsum_rows)
  int H, Hkv, V, Tmax, S, RP, tiles_per_split;
  int T_eff, last_only;                 // rows that rank: all valid text rows, or the last one alone
  float c2;                             // log2(e) / sqrt(d): accumulator units -> log2 units
  double lambda_max, eps;
  int mask_on;
};

// first text row that ranks and how many do, for image b
__device__ __forceinline__ void ranking_rows(const AttnArgs& a, int b, int& row0, int& nrows) {
  const int len = min(max(a.text_len[b], 0), a.Tmax);
  row0 = a.last_only ? max(len - 1, 0) : 0;
  nrows = a.last_only ? min(len, 1) : len;
}

// Query operands: registers (bf16) or LDS (f32, as pieces).  Operand row m is text row row0 + m; rows
// at or past nrows (padding of a ragged batch, whatever it holds) are zero operands.
template <typename T, int NRB, int NG> struct QueryOps;
template <int NRB, int NG> struct QueryOps<bf16_t, NRB, NG> {
  uint4 qa[NRB][NG];
  __device__ __forceinline__ void init(const AttnArgs& a, int b, int h, int lane, char*, int row0, int nrows) {
    const int m = lane & 31, hf = lane >> 5;
    const char* qbase = reinterpret_cast<const char*>(static_cast<const bf16_t*>(a.qt) + b * a.sq.b + h * a.sq.h +
                                                      (int64_t)row0 * a.sq.r) + hf * 16;
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
      const int row = rb * 32 + m;
#pragma unroll
      for (int c = 0; c < NG; ++c)
        qa[rb][c] = row < nrows ? ldg16(qbase + (int64_t)row * a.sq.r * 2 + c * 32) : make_uint4(0, 0, 0, 0);
    }
  }
  __device__ __forceinline__ uint4 get(int rb, int c) const { return qa[rb][c]; }
};
// f32 queries: three bf16 planes in LDS, split once per workgroup
template <int NRB, int NG> struct QueryOps<float, NRB, NG> {
  static constexpr int ROWB = NG * 32, LDSROW = ROWB + 16, PLANE = NRB * 32 * LDSROW;
  const char* base;     // the workgroup's LDS
  int qoff;             // this lane's operand row and half, as a byte offset
  __device__ __forceinline__ void init(const AttnArgs& a, int b, int h, int lane, char* lds, int row0, int nrows) {
    const char* qbase = reinterpret_cast<const char*>(static_cast<const float*>(a.qt) + b * a.sq.b + h * a.sq.h +
                                                      (int64_t)row0 * a.sq.r);
    constexpr int PPR = ROWB / 16;         // groups of 8 elements per row
#pragma unroll
    for (int i = threadIdx.x; i < NRB * 32 * PPR; i += 256) {
      int row = i / PPR, pc = i % PPR;
      Split3 s;
      s.hi = s.mid = s.lo = make_uint4(0, 0, 0, 0);
      if (row < nrows) {
        const char* p = qbase + (int64_t)row * a.sq.r * 4 + pc * 32;
        s = split_f32x8(ldg16(p), ldg16(p + 16));
      }
      char* dst = lds + row * LDSROW + pc * 16;
      *reinterpret_cast<uint4*>(dst) = s.hi;
      *reinterpret_cast<uint4*>(dst + PLANE) = s.mid;
      *reinterpret_cast<uint4*>(dst + 2 * PLANE) = s.lo;
    }
    __syncthreads();
    base = lds;
    qoff = (lane & 31) * LDSROW + (lane >> 5) * 16;
  }
  // Called once per key tile: the operands are the same for every tile, and a compiler that knew it
  // would keep all of them (12 NG NRB registers) alive across the sweep.  Only the offset is hidden
  // from it, so that the reads stay LDS reads.
  __device__ __forceinline__ void per_tile() { asm volatile("" : "+v"(qoff)); }
  __device__ __forceinline__ Split3 get3(int rb, int c) const {
    const char* p = base + qoff + rb * 32 * LDSROW + c * 32;
    Split3 s;
    s.hi = *reinterpret_cast<const uint4*>(p);
    s.mid = *reinterpret_cast<const uint4*>(p + PLANE);
    s.lo = *reinterpret_cast<const uint4*>(p + 2 * PLANE);
    return s;
  }
};
// LDS of a sweep workgroup: the f32 query pieces (two row blocks at most), then 8 x 64 floats of statistics
template <typename T, int NG> constexpr size_t query_lds_bytes() {
  return sizeof(T) == 4 ? (size_t)64 * (NG * 32 + 16) * 3 : 0;
}
constexpr int ATT_ROWS = 64;       // text rows per workgroup

// A lane's share of a 32-key tile.  bf16: the chunks are the operands.  f32: the raw chunks are split
// into pieces group by group, and a group's registers take the next tile's chunks as soon as it is split.
template <typename T, int NG> struct KeyTile;
template <int NG> struct KeyTile<bf16_t, NG> {
  uint4 op[NG];
  __device__ __forceinline__ void load(const char* krow) {
#pragma unroll
    for (int c = 0; c < NG; ++c) op[c] = ldg16(krow + c * 32);
  }
};
template <int NG> struct KeyTile<float, NG> {
  uint4 raw[2 * NG];
  __device__ __forceinline__ void load(const char* krow) {
#pragma unroll
    for (int c = 0; c < NG; ++c) load_group(krow, c);
  }
  __device__ __forceinline__ void load_group(const char* krow, int c) {
    raw[2 * c] = ldg16(krow + c * 64);
    raw[2 * c + 1] = ldg16(krow + c * 64 + 16);
  }
};

__device__ __forceinline__ float discount_of(const AttnArgs& a, double s, double lo, double inv) {
  if (!a.mask_on) return 1.0f;
  return (float)fmax(a.lambda_max * ((s - lo) * inv), a.eps);
}
__device__ __forceinline__ float discount(const AttnArgs& a, int b, int j, double lo, double inv) {
  return discount_of(a, a.mask_on ? a.s64[(int64_t)b * a.V + j] : 0.0, lo, inv);
}

// merge of two (max, sum) pairs kept in accumulator units with scale c2
__device__ __forceinline__ void merge_stat(float& m, float& s, float m2, float s2, float c2) {
  float M = fmaxf(m, m2);
  s = s * fast_exp2((m - M) * c2) + s2 * fast_exp2((m2 - M) * c2);
  m = M;
}

constexpr float ATT_NEG = -1e30f;

// online (max, sum) update of one row block from the 16 logits a lane holds
__device__ __forceinline__ void stats_update(f32x16_t& acc, const float (&lam)[16], bool ragged, int tile, int hf, int V,
                                             float c2, float& m_run, float& s_run) {
  if (ragged) {
#pragma unroll
    for (int v = 0; v < 16; ++v)
      if (tile * 32 + 8 * (v >> 2) + 4 * hf + (v & 3) >= V) acc[v] = ATT_NEG;
  }
  float mx = acc[0];
#pragma unroll
  for (int v = 1; v < 16; ++v) mx = fmaxf(mx, acc[v]);
  mx = fmaxf(mx, __shfl_xor(mx, 32));                  // both halves of the row's 32 keys
  const float m_new = fmaxf(m_run, mx);
  float s = s_run * fast_exp2((m_run - m_new) * c2);
  const float off = -m_new * c2;
#pragma unroll
  for (int v = 0; v < 16; ++v) s = fmaf(lam[v], fast_exp2(fmaf(acc[v], c2, off)), s);
  s_run = s;
  m_run = m_new;
}

// (head, row pair, key split) of a sweep workgroup
struct SweepId { int h, rp, sp, b; };
__device__ __forceinline__ SweepId sweep_id(const AttnArgs& a) {
  SweepId w;
  w.h = blockIdx.x % a.H;
  const int rest = blockIdx.x / a.H;
  w.rp = rest % a.RP;
  w.sp = rest / a.RP;
  w.b = blockIdx.y;
  return w;
}

// Keys are the tile rows here: lane (n, hf) owns text row row0 + rb*32 + n and finds, in accumulator
// register v, its logit against key 8*(v/4) + 4*hf + v%4 of the tile.
// STORE: the logits of the ranking rows are also left in zlog (row t of an image's ranking rows,
// accumulator units), so that the column sums need no second sweep over the keys.
template <typename T, int NRB, int NG, bool STORE>
__device__ __forceinline__ void attn_stats_body(const AttnArgs& a, char* lds, const SweepId& w, int row0, int nrows) {
  constexpr bool F32 = sizeof(T) == 4;
  constexpr int GB = group_bytes<T>::value;
  using Q = QueryOps<T, NRB, NG>;
  float* st_m = reinterpret_cast<float*>(lds + query_lds_bytes<T, NG>());   // [4][64]
  float* st_s = st_m + 4 * ATT_ROWS;                                         // [4][64]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, hf = lane >> 5;
  const int sp = w.sp, h = w.h, b = w.b;
  const int g = (h * a.Hkv) / a.H;
  const char* kbase = reinterpret_cast<const char*>(static_cast<const T*>(a.kv) + b * a.sk.b + g * a.sk.h) +
                      hf * GB;
  const int64_t krow_bytes = a.sk.r * (int64_t)sizeof(T);
  const int ntiles = (a.V + 31) >> 5;
  const int t_end = min(ntiles, (sp + 1) * a.tiles_per_split);
  const float c2 = a.c2;
  // the first key tile and its masses are asked for before the queries, so that the waits overlap
  KeyTile<T, NG> kb;
  int tile = sp * a.tiles_per_split + wave;
  if (tile < t_end) kb.load(kbase + (int64_t)min(tile * 32 + n, a.V - 1) * krow_bytes);
  const double* s64 = a.s64 + (int64_t)b * a.V;
  double sj = (a.mask_on && tile < t_end) ? s64[min(tile * 32 + n, a.V - 1)] : 0.0;
  Q q;
  q.init(a, b, h, lane, lds, row0, nrows);
  const double mlo = f64_unkey(a.mmkey[2 * b]), mhi = f64_unkey(a.mmkey[2 * b + 1]);
  const double minv = 1.0 / (mhi - mlo + a.eps);

  float m_run[NRB], s_run[NRB];
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) { m_run[rb] = ATT_NEG; s_run[rb] = 0.0f; }
  // where this lane's text rows start in zlog, at the lane's first key of a tile
  float* zrow[NRB];
  const bool zvec = (a.V & 3) == 0;            // rows of zlog start on 16-byte boundaries
  if constexpr (STORE) {
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
      zrow[rb] = rb * 32 + n < nrows
                     ? a.zlog + (((int64_t)b * a.H + h) * a.T_eff + w.rp * ATT_ROWS + rb * 32 + n) * a.V + 4 * hf
                     : nullptr;
  }
  auto store_logits = [&](const f32x16_t& acc, int rb, int tile, bool ragged) {
    if (zrow[rb] == nullptr) return;
    float* z = zrow[rb] + tile * 32;
    if (zvec && !ragged) {
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4*>(z + 8 * q) = make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int o = 8 * (v >> 2) + (v & 3);
        if (tile * 32 + 4 * hf + o < a.V) z[o] = acc[v];
      }
    }
  };

  for (; tile < t_end; tile += 4) {
    const int j = tile * 32 + n;
    const int tnext = tile + 4;
    const char* knext = kbase + (int64_t)min(tnext * 32 + n, a.V - 1) * krow_bytes;
    KeyTile<T, F32 ? 1 : NG> kn;      // bf16: next key tile prefetched into a second register set, first thing
    if constexpr (!F32) {
      if (tnext < t_end) kn.load(knext);
    }
    // discount of key n of the tile (its mass was asked for a tile ago), then handed to the lanes in
    // accumulator order
    const float lj = j < a.V ? discount_of(a, sj, mlo, minv) : 0.0f;
    if (a.mask_on && tnext < t_end) sj = s64[min(tnext * 32 + n, a.V - 1)];
    float lam[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) lam[v] = __shfl(lj, 8 * (v >> 2) + 4 * hf + (v & 3));
    const bool ragged = tile * 32 + 32 > a.V;
    if constexpr (!F32) {
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb) {
        f32x16_t acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
        for (int c = 0; c < NG; ++c) mma32<bf16_t>(acc, kb.op[c], q.get(rb, c));
        if constexpr (STORE) store_logits(acc, rb, tile, ragged);
        stats_update(acc, lam, ragged, tile, hf, a.V, c2, m_run[rb], s_run[rb]);
      }
      if (tnext < t_end) {
#pragma unroll
        for (int c = 0; c < NG; ++c) kb.op[c] = kn.op[c];
      }
    } else {
      // group by group: a key group is split once and meets both row blocks, whose accumulators stay
      // alive across the groups; its registers then take the same group of the next tile
      q.per_tile();
      f32x16_t acc[NRB];
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[rb][v] = 0.0f;
#pragma unroll
      for (int c = 0; c < NG; ++c) {
        const Split3 ks = split_f32x8(kb.raw[2 * c], kb.raw[2 * c + 1]);
        if (tnext < t_end) kb.load_group(knext, c);
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) mma_split(acc[rb], ks, q.get3(rb, c));
      }
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb) {
        if constexpr (STORE) store_logits(acc[rb], rb, tile, ragged);
        stats_update(acc[rb], lam, ragged, tile, hf, a.V, c2, m_run[rb], s_run[rb]);
      }
    }
  }
  // the two halves of a wave share the row maximum: their sums just add; then the 4 waves
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    float s = s_run[rb] + __shfl_xor(s_run[rb], 32);
    if (hf == 0) {
      st_m[wave * ATT_ROWS + rb * 32 + n] = m_run[rb];
      st_s[wave * ATT_ROWS + rb * 32 + n] = s;
    }
  }
  __syncthreads();
  if (tid < NRB * 32) {
    float m = st_m[tid], s = st_s[tid];
    for (int wv = 1; wv < 4; ++wv) merge_stat(m, s, st_m[wv * ATT_ROWS + tid], st_s[wv * ATT_ROWS + tid], c2);
    const int NR = ATT_ROWS * a.RP;
    float* out = a.pstat + ((((int64_t)b * a.H + h) * a.S + sp) * 2) * NR + w.rp * ATT_ROWS;
    out[tid] = m;
    out[NR + tid] = s;
  }
}

template <typename T, int NG, bool STORE>
__global__ __launch_bounds__(256, 2) void k_attn_stats(AttnArgs a) {
  extern __shared__ __align__(16) char lds[];
  const SweepId w = sweep_id(a);
  int row0, nrows;
  ranking_rows(a, w.b, row0, nrows);
  row0 += w.rp * ATT_ROWS;
  nrows = min(nrows - w.rp * ATT_ROWS, ATT_ROWS);
  if (nrows <= 0) return;                      // the image's text ends before this pair of row blocks
  if (nrows <= 32) attn_stats_body<T, 1, NG, STORE>(a, lds, w, row0, nrows);
  else attn_stats_body<T, 2, NG, STORE>(a, lds, w, row0, nrows);
}

// Row statistics merged over the splits, with the rest of the row (lse_extra) folded in: per text
// row -max (log2 units) and 1 / denominator; rows that do not rank get (-inf, 0) so that they add
// nothing.  Threads tid < n_local of the workgroup handle rows first + tid of the NR-row layout;
// row0 = the text row of local row 0; fin_o / fin_i in LDS.
__device__ __forceinline__ void final_row_stats(const AttnArgs& a, int b, int h, int NR, int first, int n_local,
                                                int row0, int nrows, float* fin_o, float* fin_i) {
  const int tid = threadIdx.x;
  if (tid < n_local) {
    const bool row_ok = tid < nrows;
    float o = -INFINITY, iv = 0.0f;        // 2^(z - inf) = 0: rows that do not rank add nothing
    if (row_ok) {
      const float* ps = a.pstat + (((int64_t)b * a.H + h) * a.S * 2) * NR + first;
      float m = ps[tid], s = ps[NR + tid];
      for (int wv = 1; wv < a.S; ++wv) merge_stat(m, s, ps[(wv * 2) * NR + tid], ps[(wv * 2 + 1) * NR + tid], a.c2);
      float m2 = m * a.c2;                                           // log2 units from here on
      if (a.lse_extra != nullptr) {
        float l2 = a.lse_extra[((int64_t)b * a.H + h) * a.Tmax + row0 + tid] * 1.4426950408889634f;
        float M = fmaxf(m2, l2);
        s = s * fast_exp2(m2 - M) + fast_exp2(l2 - M);
        m2 = M;
      }
      o = -m2;
      iv = 1.0f / s;
    }
    fin_o[tid] = o;
    fin_i[tid] = iv;
  }
}

// Queries are the tile rows here: lane (n, hf) owns key n of the tile and finds, in accumulator
// register v of row block rb, its logit against text row row0 + rb*32 + 8*(v/4) + 4*hf + v%4.
template <typename T, int NRB, int NG>
__device__ __forceinline__ void attn_colsum_body(const AttnArgs& a, char* lds, const SweepId& w, int row0, int nrows) {
  constexpr bool F32 = sizeof(T) == 4;
  constexpr int GB = group_bytes<T>::value;
  using Q = QueryOps<T, NRB, NG>;
  float* fin_o = reinterpret_cast<float*>(lds + query_lds_bytes<T, NG>());   // [64]  -max * c2
  float* fin_i = fin_o + ATT_ROWS;                                            // [64]  1 / denominator
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, hf = lane >> 5;
  const int sp = w.sp, h = w.h, b = w.b;
  const int g = (h * a.Hkv) / a.H;
  const float c2 = a.c2;
  const char* kbase = reinterpret_cast<const char*>(static_cast<const T*>(a.kv) + b * a.sk.b + g * a.sk.h) +
                      hf * GB;
  const int64_t krow_bytes = a.sk.r * (int64_t)sizeof(T);
  const int ntiles = (a.V + 31) >> 5;
  const int t_end = min(ntiles, (sp + 1) * a.tiles_per_split);
  // the first key tile is asked for before the statistics and the queries, so that the waits overlap
  KeyTile<T, NG> kb;
  int tile = sp * a.tiles_per_split + wave;
  if (tile < t_end) kb.load(kbase + (int64_t)min(tile * 32 + n, a.V - 1) * krow_bytes);
  final_row_stats(a, b, h, ATT_ROWS * a.RP, w.rp * ATT_ROWS, NRB * 32, row0, nrows, fin_o, fin_i);
  Q q;
  q.init(a, b, h, lane, lds, row0, nrows);
  __syncthreads();
  // bf16: the row statistics of the 16 rows a lane meets stay in registers; f32 (whose registers go to
  // the key pieces and to the accumulators) reads them from LDS after the products
  constexpr int NST = F32 ? 1 : NRB;
  float off[NST][16], inv[NST][16];
  if constexpr (!F32) {
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        int row = rb * 32 + mma32_row(v, lane);
        off[rb][v] = fin_o[row];
        inv[rb][v] = fin_i[row];
      }
  }
  float* out = a.upart + (((int64_t)b * a.H + h) * a.RP + w.rp) * a.V;
  for (; tile < t_end; tile += 4) {
    const int j = tile * 32 + n;
    const int tnext = tile + 4;
    const char* knext = kbase + (int64_t)min(tnext * 32 + n, a.V - 1) * krow_bytes;
    float u = 0.0f;
    if constexpr (!F32) {
      KeyTile<T, NG> kn;
      if (tnext < t_end) kn.load(knext);
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb) {
        f32x16_t acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
        for (int c = 0; c < NG; ++c) mma32<bf16_t>(acc, q.get(rb, c), kb.op[c]);
#pragma unroll
        for (int v = 0; v < 16; ++v) u = fmaf(fast_exp2(fmaf(acc[v], c2, off[rb][v])), inv[rb][v], u);
      }
      if (tnext < t_end) {
#pragma unroll
        for (int c = 0; c < NG; ++c) kb.op[c] = kn.op[c];
      }
    } else {
      q.per_tile();
      f32x16_t acc[NRB];
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[rb][v] = 0.0f;
#pragma unroll
      for (int c = 0; c < NG; ++c) {
        const Split3 ks = split_f32x8(kb.raw[2 * c], kb.raw[2 * c + 1]);
        if (tnext < t_end) kb.load_group(knext, c);
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) mma_split(acc[rb], q.get3(rb, c), ks);
      }
      int fz = 0;
      asm volatile("" : "+v"(fz));       // re-read per tile rather than kept in 32 NRB registers
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = fz + rb * 32 + mma32_row(v, lane);
          u = fmaf(fast_exp2(fmaf(acc[rb][v], c2, fin_o[row])), fin_i[row], u);
        }
    }
    u += __shfl_xor(u, 32);
    if (hf == 0 && j < a.V) out[j] = u;
  }
}

template <typename T, int NG>
__global__ __launch_bounds__(256, 2) void k_attn_colsum(AttnArgs a) {
  extern __shared__ __align__(16) char lds[];
  const SweepId w = sweep_id(a);
  int row0, nrows;
  ranking_rows(a, w.b, row0, nrows);
  row0 += w.rp * ATT_ROWS;
  nrows = min(nrows - w.rp * ATT_ROWS, ATT_ROWS);
  if (nrows <= 0) {
    // the image's text ends before this pair of row blocks: its column sums are zero
    const int ntiles = (a.V + 31) >> 5;
    const int j_lo = w.sp * a.tiles_per_split * 32, j_hi = min(a.V, min(ntiles, (w.sp + 1) * a.tiles_per_split) * 32);
    float* out = a.upart + (((int64_t)w.b * a.H + w.h) * a.RP + w.rp) * a.V;
    for (int j = j_lo + threadIdx.x; j < j_hi; j += 256) out[j] = 0.0f;
    return;
  }
  if (nrows <= 32) attn_colsum_body<T, 1, NG>(a, lds, w, row0, nrows);
  else attn_colsum_body<T, 2, NG>(a, lds, w, row0, nrows);
}

// ------------------------------------------------------------------------------------------
// The same two reductions from stored logits zlog [B, H, T_eff, V] (accumulator units), for the
// text rows that rode in the mass sweep.
// k_rowstats_logits: grid (T_eff, H, B), 256 threads: (max, sum of lambda'_j 2^z) of one row, in the
// layout k_attn_stats leaves (one split, 32 rows per block).
// k_colsum_logits: grid (ceil(V / 256), H, B), 256 threads: normalised column sums per key.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_rowstats_logits(AttnArgs a) {
  __shared__ float red_m[4], red_s[4];
  const int t = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int row0, nrows;
  ranking_rows(a, b, row0, nrows);
  if (t >= nrows) return;                                   // uniform for the workgroup
  const double mlo = f64_unkey(a.mmkey[2 * b]), mhi = f64_unkey(a.mmkey[2 * b + 1]);
  const double minv = 1.0 / (mhi - mlo + a.eps);
  const float* z = a.zlog + (((int64_t)b * a.H + h) * a.T_eff + t) * a.V;
  float m = ATT_NEG;
  for (int j = tid; j < a.V; j += 256) m = fmaxf(m, z[j]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
  if (lane == 0) red_m[wave] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));
  const float offv = -m * a.c2;
  float s = 0.0f;
  for (int j = tid; j < a.V; j += 256) s = fmaf(discount(a, b, j, mlo, minv), fast_exp2(fmaf(z[j], a.c2, offv)), s);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
  if (lane == 0) red_s[wave] = s;
  __syncthreads();
  if (tid == 0) {
    const int NR = ((a.T_eff + 31) >> 5) * 32;
    float* out = a.pstat + (((int64_t)b * a.H + h) * 2) * NR;     // one split
    out[t] = m;
    out[NR + t] = (red_s[0] + red_s[1]) + (red_s[2] + red_s[3]);
  }
}

__global__ __launch_bounds__(256) void k_colsum_logits(AttnArgs a) {
  __shared__ float fin_o[32], fin_i[32];
  const int h = blockIdx.y, b = blockIdx.z;
  const int j = blockIdx.x * 256 + threadIdx.x;
  int row0, nrows;
  ranking_rows(a, b, row0, nrows);
  final_row_stats(a, b, h, 32, 0, 32, row0, nrows, fin_o, fin_i);
  __syncthreads();
  if (j >= a.V) return;
  const float* z = a.zlog + (((int64_t)b * a.H + h) * a.T_eff) * a.V + j;
  float u = 0.0f;
  for (int t = 0; t < nrows; ++t) u = fmaf(fast_exp2(fmaf(z[(int64_t)t * a.V], a.c2, fin_o[t])), fin_i[t], u);
  a.upart[((int64_t)b * a.H + h) * a.V + j] = u;
}

// Column sums from the logits k_attn_stats<.., true> left: grid (ceil(V / 256), H, B), 256 threads.
// A lane takes four neighbouring keys, the four waves take the ranking rows t = wave, wave + 4, ...
// (256 at a time: their statistics sit in LDS), and the waves' partial sums are added in wave order.
// upart then has one row per head.
__global__ __launch_bounds__(256) void k_colsum_rows(AttnArgs a) {
  __shared__ float fin_o[256], fin_i[256];
  __shared__ float4 part[4][64];
  const int h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j0 = blockIdx.x * 256 + lane * 4;
  int row0, nrows;
  ranking_rows(a, b, row0, nrows);
  const int NR = ATT_ROWS * a.RP;
  const bool vec = (a.V & 3) == 0;
  const float* z = a.zlog + (((int64_t)b * a.H + h) * a.T_eff) * a.V + j0;
  const float c2 = a.c2;
  float4 u = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  for (int first = 0; first < nrows; first += 256) {
    if (first) __syncthreads();
    final_row_stats(a, b, h, NR, first, min(256, NR - first), row0 + first, nrows - first, fin_o, fin_i);
    __syncthreads();
    const int nl = min(256, nrows - first);
    if (j0 < a.V) {
#pragma unroll 4
      for (int t = wave; t < nl; t += 4) {
        const float* zr = z + (int64_t)(first + t) * a.V;
        float4 x;
        if (vec) {
          x = *reinterpret_cast<const float4*>(zr);
        } else {
          x.x = zr[0];
          x.y = j0 + 1 < a.V ? zr[1] : 0.0f;
          x.z = j0 + 2 < a.V ? zr[2] : 0.0f;
          x.w = j0 + 3 < a.V ? zr[3] : 0.0f;
        }
        const float o = fin_o[t], iv = fin_i[t];
        u.x = fmaf(fast_exp2(fmaf(x.x, c2, o)), iv, u.x);
        u.y = fmaf(fast_exp2(fmaf(x.y, c2, o)), iv, u.y);
        u.z = fmaf(fast_exp2(fmaf(x.z, c2, o)), iv, u.z);
        u.w = fmaf(fast_exp2(fmaf(x.w, c2, o)), iv, u.w);
      }
    }
  }
  part[wave][lane] = u;
  __syncthreads();
  if (wave == 0 && j0 < a.V) {
    float4 r = part[0][lane];
#pragma unroll
    for (int wv = 1; wv < 4; ++wv) {
      const float4 q = part[wv][lane];
      r.x += q.x; r.y += q.y; r.z += q.z; r.w += q.w;
    }
    float* out = a.upart + ((int64_t)b * a.H + h) * a.V + j0;
    if (vec) {
      *reinterpret_cast<float4*>(out) = r;
    } else {
      out[0] = r.x;
      if (j0 + 1 < a.V) out[1] = r.y;
      if (j0 + 2 < a.V) out[2] = r.z;
      if (j0 + 3 < a.V) out[3] = r.w;
    }
  }
}

// ------------------------------------------------------------------------------------------
// k_score: grid (ceil(V/64), B), 256 threads: 64 keys x 4 head groups.  rows[b] = text rows that
// ranked (the divisor of the mean).
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ double rank_count(const int32_t* text_len, int b, int Tmax, int last_only) {
  const int len = min(max(text_len[b], 0), Tmax);
  return (double)(last_only ? min(len, 1) : len);
}

__global__ __launch_bounds__(256) void k_score(const float* __restrict__ upart, const double* __restrict__ s64,
                                                const unsigned long long* __restrict__ mmkey,
                                                const int32_t* __restrict__ text_len, int H, int HV, int V, int Tmax,
                                                int last_only, double lambda_max, double eps, int mask_on,
                                                float* __restrict__ s_hat, float* __restrict__ score) {
  // HV = rows of upart per image: one per head and pair of text-row blocks
  __shared__ double part[4][64];
  const int b = blockIdx.y, jl = threadIdx.x & 63, hq = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + jl;
  double u = 0.0;
  if (j < V) {
    const float* up = upart + (int64_t)b * HV * V + j;
    int h = hq;
    for (; h + 12 < HV; h += 16) {
      float u0 = up[(int64_t)h * V], u1 = up[(int64_t)(h + 4) * V], u2 = up[(int64_t)(h + 8) * V],
            u3 = up[(int64_t)(h + 12) * V];
      u += (double)u0;
      u += (double)u1;
      u += (double)u2;
      u += (double)u3;
    }
    for (; h < HV; h += 4) u += (double)up[(int64_t)h * V];
  }
  part[hq][jl] = u;
  __syncthreads();
  if (hq == 0 && j < V) {
    u = ((part[0][jl] + part[1][jl]) + part[2][jl]) + part[3][jl];
    const double lo = f64_unkey(mmkey[2 * b]), hi = f64_unkey(mmkey[2 * b + 1]);
    const double sh = (s64[(int64_t)b * V + j] - lo) * (1.0 / (hi - lo + eps));
    const double lam = mask_on ? fmax(lambda_max * sh, eps) : 1.0;
    s_hat[(int64_t)b * V + j] = (float)sh;
    score[(int64_t)b * V + j] = (float)(lam * u / ((double)H * rank_count(text_len, b, Tmax, last_only)));
  }
}

// ------------------------------------------------------------------------------------------
// k_score_select: grid (B), 1024 threads, dynamic LDS = V floats when V > 1024.  The threads reduce the
// per-head column sums of the keys tid, tid + 1024, ... (coalesced) in the order k_score uses (four
// interleaved head groups in fp64, then ((0+1)+2)+3), so that score and s_hat come out bit-identical to
// k_score's; the scores change hands through LDS to the blocked layout of the selection (thread t owns
// keys t*ipt .. t*ipt+ipt-1), and the workgroup then selects exactly as k_select does.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void score_select_image(const int b, const float* __restrict__ upart,
                                                   const double* __restrict__ s64,
                                                   const unsigned long long* __restrict__ mmkey,
                                                   const int32_t* __restrict__ text_len, int H, int HV, int V, int k,
                                                   int Tmax, int last_only, double lambda_max, double eps, int mask_on,
                                                   float* __restrict__ s_hat, float* __restrict__ score,
                                                   int32_t* __restrict__ kept, int32_t* __restrict__ pruned) {
  __shared__ SelectShared sh;
  extern __shared__ float sc_lds[];
  const int tid = threadIdx.x;
  const int ipt = (V + SEL_THREADS - 1) / SEL_THREADS;
  const int i0 = tid * ipt;
  const double lo = f64_unkey(mmkey[2 * b]), hi = f64_unkey(mmkey[2 * b + 1]);
  const double inv = 1.0 / (hi - lo + eps);
  const double norm = (double)H * rank_count(text_len, b, Tmax, last_only);
  const float* up = upart + (int64_t)b * HV * V;
  float mine = 0.0f;
  for (int j = tid; j < V; j += SEL_THREADS) {
    double part[4] = {0.0, 0.0, 0.0, 0.0};
    int h = 0;
    for (; h + 16 <= HV; h += 16) {         // 16 loads in flight; row h adds to group h % 4, in order
      float u[16];
#pragma unroll
      for (int q = 0; q < 16; ++q) u[q] = up[(int64_t)(h + q) * V + j];
#pragma unroll
      for (int q = 0; q < 16; ++q) part[q & 3] += (double)u[q];
    }
    for (; h < HV; ++h) part[h & 3] += (double)up[(int64_t)h * V + j];
    const double usum = ((part[0] + part[1]) + part[2]) + part[3];
    const double shat = (s64[(int64_t)b * V + j] - lo) * inv;
    const double lam = mask_on ? fmax(lambda_max * shat, eps) : 1.0;
    const float sc = (float)(lam * usum / norm);
    s_hat[(int64_t)b * V + j] = (float)shat;
    score[(int64_t)b * V + j] = sc;
    if (ipt > 1) sc_lds[j] = sc;
    else mine = sc;
  }
  if (ipt > 1) __syncthreads();
  uint32_t key[SEL_IPT];
#pragma unroll
  for (int e = 0; e < SEL_IPT; ++e) {
    const int i = i0 + e;
    key[e] = (e < ipt && i < V) ? float_key(ipt > 1 ? sc_lds[i] : mine) : 0u;
  }
  int n_keep;
  const uint32_t keep_bits = radix_topk(key, ipt, i0, V, k, sh, &n_keep);
  int tot;
  int kept_before = block_scan_excl(n_keep, sh.wave_sums, &tot);
  int32_t* kout = kept + (int64_t)b * k;
  int32_t* pout = pruned + (int64_t)b * (V - k);
#pragma unroll
  for (int e = 0; e < SEL_IPT; ++e) {
    const int i = i0 + e;
    if (e < ipt && i < V) {
      if (keep_bits & (1u << e)) kout[kept_before++] = i;
      else pout[i - kept_before] = i;
    }
  }
}

__global__ __launch_bounds__(SEL_THREADS) void k_score_select(const float* __restrict__ upart,
                                                               const double* __restrict__ s64,
                                                               const unsigned long long* __restrict__ mmkey,
                                                               const int32_t* __restrict__ text_len, int H, int HV,
                                                               int V, int k, int Tmax, int last_only, double lambda_max,
                                                               double eps, int mask_on, float* __restrict__ s_hat,
                                                               float* __restrict__ score, int32_t* __restrict__ kept,
                                                               int32_t* __restrict__ pruned) {
  score_select_image(blockIdx.x, upart, s64, mmkey, text_len, H, HV, V, k, Tmax, last_only, lambda_max, eps, mask_on,
                     s_hat, score, kept, pruned);
}

// k_score_select_kv: grid (B + n_bufs * B * Hkv).  The first B workgroups are k_score_select's.  Each of the
// others copies, for one (cache buffer, image, kv head), the rows that survive whatever is selected
// (Fig. 3: prefix rows stay where they are, valid text row t moves from P + V + t to P + k + t): they
// depend on no result of the stage, and the B selecting workgroups leave the memory system idle.
// A row is row_bytes / 16 pieces of 16 bytes; two rows per thread are in flight.
__global__ __launch_bounds__(SEL_THREADS) void k_score_select_kv(
    const float* __restrict__ upart, const double* __restrict__ s64, const unsigned long long* __restrict__ mmkey,
    const int32_t* __restrict__ text_len, int H, int HV, int V, int k, int Tmax, int last_only, double lambda_max,
    double eps, int mask_on, float* __restrict__ s_hat, float* __restrict__ score, int32_t* __restrict__ kept,
    int32_t* __restrict__ pruned, int B, KvFixedRows fx) {
  if ((int)blockIdx.x < B) {
    score_select_image(blockIdx.x, upart, s64, mmkey, text_len, H, HV, V, k, Tmax, last_only, lambda_max, eps,
                       mask_on, s_hat, score, kept, pruned);
    return;
  }
  const int gid = blockIdx.x - B, groups = B * fx.Hkv;
  const int buf = gid / groups, bg = gid % groups, b = bg / fx.Hkv;
  const int lpr = fx.row_bytes >> 4, rpi = SEL_THREADS / lpr;
  const int tid = threadIdx.x, piece = tid % lpr, r0 = tid / lpr;
  const int n_fixed = fx.P + min(max(text_len[b], 0), fx.Tmax);
  const char* src = fx.ptrs.src[buf] + (int64_t)bg * fx.N * fx.row_bytes + piece * 16;
  char* dst = fx.ptrs.dst[buf] + (int64_t)bg * fx.Nout * fx.row_bytes + piece * 16;
  for (int r = r0; r < n_fixed; r += 2 * rpi) {
    const int r2 = r + rpi;
    const int sa = r < fx.P ? r : r + fx.V, da = r < fx.P ? r : r + fx.k;
    const int sb = r2 < fx.P ? r2 : r2 + fx.V, db = r2 < fx.P ? r2 : r2 + fx.k;
    const uint4 va = ldg16_stream(src + (int64_t)sa * fx.row_bytes);
    uint4 vb = va;
    if (r2 < n_fixed) vb = ldg16_stream(src + (int64_t)sb * fx.row_bytes);
    stg16_stream(dst + (int64_t)da * fx.row_bytes, va);
    if (r2 < n_fixed) stg16_stream(dst + (int64_t)db * fx.row_bytes, vb);
  }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
static int ranking_rows_max(const asap_params& p) { return p.score_rows == ASAP_ROWS_LAST ? 1 : p.Tmax; }

// Key-range splits of the two text-row sweeps.  Their workgroups run in rounds of as many as fit
// on the chip at once (1 to 4 per compute unit, by the registers of the instantiation); a round
// costs the tiles of one split plus a fixed part (start-up, the text queries, the last tiles' tail:
// about 8 tile times, fitted to measurements), and more than one workgroup per compute unit at a
// time slows each of them (about 1.4x).  The count with the least modelled time wins, fewer splits
// on ties; a split has at least 4 tiles (one per wave).
static int attn_splits(const asap_params& p) {
  const int ntiles = (p.V + 31) / 32;
  const int rows = ranking_rows_max(p);
  const int rb = rows > 32 ? 2 : 1, ch = p.d / 16, rp = (rows + 63) / 64;
  int per_cu = rb * ch <= 4 ? 4 : (rb * ch <= 8 && ch == 8) ? 3 : 2;
  if (p.qk_dtype != ASAP_BF16) per_cu = 2;
  const long slots = 256L * per_cu, groups = (long)p.H * p.B * rp;
  int smax = ntiles / 4;
  if (smax > 16) smax = 16;
  if (smax < 1) smax = 1;
  int best = 1;
  double best_cost = -1.0;
  for (int s = 1; s <= smax; ++s) {
    const int tps = (ntiles + s - 1) / s;
    if ((ntiles + tps - 1) / tps != s) continue;           // the same split length with fewer splits exists
    const long wgs = groups * s, rounds = (wgs + slots - 1) / slots;
    const double crowd = (wgs < slots ? wgs : slots) <= 256 ? 1.0 : 1.4;
    const double cost = (double)rounds * (tps + 8) * crowd;
    if (best_cost < 0.0 || cost < best_cost) { best_cost = cost; best = s; }
  }
  return best;
}

ScoreWorkspace score_workspace(const asap_params& p, size_t budget) {
  ScoreWorkspace w;
  // rows per k_qsum block: whole image span unless that leaves the chip short of blocks
  int chunks = (512 + p.B * p.H - 1) / (p.B * p.H);
  if (chunks > (p.V + 255) / 256) chunks = (p.V + 255) / 256;
  if (chunks < 1) chunks = 1;
  w.q_rows = (p.V + chunks - 1) / chunks;
  w.q_chunks = (p.V + w.q_rows - 1) / w.q_rows;
  w.attn_splits = attn_splits(p);
  w.t_eff = ranking_rows_max(p);
  // Text rows ride in the mass sweep when the rows of one kv head's query heads fit the free rows of
  // its tile and their logits -- written once, read twice, 12 bytes per row and key -- weigh less than
  // the two sweeps over the keys they replace.
  const int G = p.H / p.Hkv, rows = G * w.t_eff;
  const int row_bytes = p.d * (p.qk_dtype == ASAP_BF16 ? 2 : 4);
  w.ride = (p.qk_dtype == ASAP_BF16 && rows <= 28 && 12 * rows < 2 * row_bytes) ? 1 : 0;
  // kv-head groups of the mass sweep: 1 unless the key tiles alone leave most of the chip idle
  const long tiles = (long)((p.V + 31) / 32) * p.B;
  w.head_splits = 1;
  if (tiles < 256) {
    int want = (int)((512 + tiles - 1) / tiles);
    for (int hs = p.Hkv; hs >= 1; --hs)
      if (p.Hkv % hs == 0 && hs <= want) { w.head_splits = hs; break; }
  }
  w.row_pairs = w.ride ? 1 : (w.t_eff + 63) / 64;
  // f32 keys: the first text-row sweep leaves its logits (4 bytes per ranking row and key, never more
  // than the key sweeps they replace at 512 bytes per key and 64 rows) and the column sums read them
  // back instead of sweeping the keys and forming the products again, as long as the workspace stays
  // moderate.
  const size_t zlog_bytes = sizeof(float) * (size_t)p.B * p.H * w.t_eff * p.V;
  w.store_logits = (!w.ride && p.qk_dtype != ASAP_BF16 && zlog_bytes <= STORED_LOGITS_MAX_BYTES) ? 1 : 0;
  const int NR = w.ride ? 32 : 64 * w.row_pairs;
  const int splits = w.ride ? 1 : w.attn_splits;
  size_t off = 0;
  w.off_qpart = off;  off = align256(off + sizeof(double) * p.B * p.H * w.q_chunks * p.d);
  w.off_qbar = off;   off = align256(off + sizeof(double) * p.B * p.Hkv * p.d);
  w.off_qsplit = off; off = align256(off + sizeof(uint16_t) * p.B * p.Hkv * 4 * p.d);
  w.off_s64 = off;    off = align256(off + sizeof(double) * p.B * p.V);
  w.off_mm = off;     off = align256(off + sizeof(double) * p.B * 2);
  w.off_pstat = off;  off = align256(off + sizeof(float) * (size_t)p.B * p.H * splits * 2 * NR);
  w.off_upart = off;  off = align256(off + sizeof(float) * (size_t)p.B * p.H * w.row_pairs * p.V);
  w.off_spart = off;
  if (w.head_splits > 1) off = align256(off + sizeof(double) * (size_t)w.head_splits * p.B * p.V);
  w.off_zlog = off;
  if (w.store_logits && align256(off + zlog_bytes) > budget) w.store_logits = 0;
  if (w.ride || w.store_logits) off = align256(off + zlog_bytes);
  w.total = off;
  return w;
}

template <typename T, int NG>
static hipError_t launch_attn(const asap_params& p, const AttnArgs& a, bool store_logits, hipStream_t st,
                              Timer* tm) {
  const size_t lds = query_lds_bytes<T, NG>() + sizeof(float) * 8 * ATT_ROWS;
  const dim3 grid(p.H * a.RP * a.S, p.B);
  if constexpr (sizeof(T) == 4) {
    if (store_logits) {
      auto ks = k_attn_stats<T, NG, true>;
      if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(ks),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
      }
      ASAP_LAUNCH(tm, "k_attn_stats", ks, grid, dim3(256), lds, st, a);
      ASAP_LAUNCH(tm, "k_colsum_rows", k_colsum_rows, dim3((p.V + 255) / 256, p.H, p.B), dim3(256), 0, st, a);
      return hipGetLastError();
    }
  }
  auto k1 = k_attn_stats<T, NG, false>;
  auto k2 = k_attn_colsum<T, NG>;
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k1),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(k2), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)lds);
    if (e != hipSuccess) return e;
  }
  ASAP_LAUNCH(tm, "k_attn_stats", k1, grid, dim3(256), lds, st, a);
  ASAP_LAUNCH(tm, "k_attn_colsum", k2, grid, dim3(256), lds, st, a);
  return hipGetLastError();
}

template <typename T, int NG>
static hipError_t launch_mass(const asap_params& p, const ScoreWorkspace& w, const void* k_vis, Strides3 kv,
                              const uint16_t* qsplit, double scale, double* s64, float* s_raw,
                              unsigned long long* mmkey, double* spart, const RideArgs& ra, hipStream_t st,
                              Timer* tm) {
  const int ktiles = (p.V + 31) / 32;
  const dim3 grid(ktiles, p.B * w.head_splits);
  const T* kp = static_cast<const T*>(k_vis);
  if constexpr (sizeof(T) == 2) {
    if (w.ride) {
      ASAP_LAUNCH(tm, "k_mass_mfma", (k_mass_mfma<T, NG, true>), grid, dim3(256), 0, st, kp, kv, qsplit, p.Hkv, p.V,
                  w.head_splits, scale, s64, s_raw, mmkey, spart, ra);
      return hipGetLastError();
    }
  }
  ASAP_LAUNCH(tm, "k_mass_mfma", (k_mass_mfma<T, NG, false>), grid, dim3(256), 0, st, kp, kv, qsplit, p.Hkv, p.V,
              w.head_splits, scale, s64, s_raw, mmkey, spart, ra);
  return hipGetLastError();
}

template <typename T>
static hipError_t score_typed(const asap_params& p, const void* q_vis, Strides3 qv, const void* q_txt,
                              Strides3 qt, const void* k_vis, Strides3 kv, const int32_t* text_len,
                              const float* lse_extra, float* s_raw, float* s_hat, float* score, int32_t* kept,
                              int32_t* pruned, const FrontArgs* fe, const KvFixedRows* fixed, char* ws,
                              size_t ws_budget, hipStream_t st, Timer* tm) {
  const ScoreWorkspace w = score_workspace(p, ws_budget);
  double* qpart = reinterpret_cast<double*>(ws + w.off_qpart);
  double* qbar = reinterpret_cast<double*>(ws + w.off_qbar);
  uint16_t* qsplit = reinterpret_cast<uint16_t*>(ws + w.off_qsplit);
  double* s64 = reinterpret_cast<double*>(ws + w.off_s64);
  unsigned long long* mmkey = reinterpret_cast<unsigned long long*>(ws + w.off_mm);
  float* pstat = reinterpret_cast<float*>(ws + w.off_pstat);
  float* upart = reinterpret_cast<float*>(ws + w.off_upart);
  double* spart = reinterpret_cast<double*>(ws + w.off_spart);
  float* zlog = reinterpret_cast<float*>(ws + w.off_zlog);
  const int mask_on = p.mask_mode == ASAP_MASK_KEYBIAS;
  const int last_only = p.score_rows == ASAP_ROWS_LAST;
  const int ng = p.d / 16;      // contraction groups of 8 elements per lane half
  const int ktiles = (p.V + 31) / 32;

  if (fe != nullptr) {
    // the summed visual queries come from the hidden states (asap_front.hip), one chunk per head
    hipError_t e0 = launch_front_end(p, fe->hidden, fe->hsb, fe->hsr, fe->wq, fe->rope_theta, fe->vis_positions,
                                     qpart, fe->ws, st, tm);
    if (e0 != hipSuccess) return e0;
    ASAP_LAUNCH(tm, "k_qsplit", k_qsplit, dim3(p.Hkv, p.B), dim3(p.d), 0, st, qpart, qbar, qsplit, p.H, p.Hkv, 1, p.d,
                mmkey);
  } else {
    const int direct = (w.q_chunks == 1 && p.H == p.Hkv) ? 1 : 0;
    ASAP_LAUNCH(tm, "k_qsum", k_qsum<T>, dim3(w.q_chunks, p.H, p.B), dim3(1024), 0, st, static_cast<const T*>(q_vis),
                qv, p.V, p.d, w.q_rows, qpart, mmkey, qbar, qsplit, direct);
    if (!direct)
      ASAP_LAUNCH(tm, "k_qsplit", k_qsplit, dim3(p.Hkv, p.B), dim3(p.d), 0, st, qpart, qbar, qsplit, p.H, p.Hkv,
                  w.q_chunks, p.d, mmkey);
  }
  const double scale = 1.0 / ((double)p.H * sqrt((double)p.d));
  RideArgs ra;
  ra.qt = q_txt; ra.sq = qt; ra.text_len = text_len; ra.zlog = zlog;
  ra.H = p.H; ra.G = p.H / p.Hkv; ra.T_eff = w.t_eff; ra.Tmax = p.Tmax; ra.last_only = last_only;
  hipError_t e = ng == 8 ? launch_mass<T, 8>(p, w, k_vis, kv, qsplit, scale, s64, s_raw, mmkey, spart, ra, st, tm)
                         : launch_mass<T, 4>(p, w, k_vis, kv, qsplit, scale, s64, s_raw, mmkey, spart, ra, st, tm);
  if (e != hipSuccess) return e;
  if (w.head_splits > 1)
    ASAP_LAUNCH(tm, "k_mass_finish", k_mass_finish, dim3(p.B), dim3(1024), 0, st, spart, w.head_splits, p.B, p.V,
                scale, s64, s_raw, mmkey);

  AttnArgs a;
  a.qt = q_txt; a.sq = qt; a.kv = k_vis; a.sk = kv; a.s64 = s64; a.mmkey = mmkey; a.text_len = text_len;
  a.lse_extra = lse_extra; a.pstat = pstat; a.upart = upart; a.zlog = zlog;
  a.H = p.H; a.Hkv = p.Hkv; a.V = p.V; a.Tmax = p.Tmax; a.S = w.ride ? 1 : w.attn_splits; a.RP = w.row_pairs;
  a.tiles_per_split = (ktiles + a.S - 1) / a.S;
  a.T_eff = w.t_eff; a.last_only = last_only;
  a.c2 = (float)(1.4426950408889634 / sqrt((double)p.d));
  a.lambda_max = (double)p.lambda_max; a.eps = (double)p.eps; a.mask_on = mask_on;
  if (w.ride) {
    ASAP_LAUNCH(tm, "k_rowstats_logits", k_rowstats_logits, dim3(w.t_eff, p.H, p.B), dim3(256), 0, st, a);
    ASAP_LAUNCH(tm, "k_colsum_logits", k_colsum_logits, dim3((p.V + 255) / 256, p.H, p.B), dim3(256), 0, st, a);
    e = hipGetLastError();
  } else if (ng == 8) {
    e = launch_attn<T, 8>(p, a, w.store_logits != 0, st, tm);
  } else {
    e = launch_attn<T, 4>(p, a, w.store_logits != 0, st, tm);
  }
  if (e != hipSuccess) return e;
  const int u_rows = p.H * (w.store_logits ? 1 : w.row_pairs);     // rows of upart per image
  if (kept != nullptr && !score_fuses_selection(p)) {
    ASAP_LAUNCH(tm, "k_score", k_score, dim3((p.V + 63) / 64, p.B), dim3(256), 0, st, upart, s64, mmkey, text_len,
                p.H, u_rows, p.V, p.Tmax, last_only, (double)p.lambda_max, (double)p.eps, mask_on, s_hat, score);
    hipError_t e2 = hipGetLastError();
    return e2 != hipSuccess ? e2 : launch_select(p, score, kept, pruned, st, tm);
  }
  if (kept != nullptr) {
    const size_t lds = p.V > SEL_THREADS ? sizeof(float) * (size_t)p.V : 0;
    const void* fn = fixed ? reinterpret_cast<const void*>(k_score_select_kv)
                           : reinterpret_cast<const void*>(k_score_select);
    if (lds > 32 * 1024) {
      e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
    }
    if (fixed)
      ASAP_LAUNCH(tm, "k_score_select_kv", k_score_select_kv, dim3(p.B + fixed->n_bufs * p.B * p.Hkv),
                  dim3(SEL_THREADS), lds, st, upart, s64, mmkey, text_len, p.H, u_rows, p.V, p.k, p.Tmax,
                  last_only, (double)p.lambda_max, (double)p.eps, mask_on, s_hat, score, kept, pruned, p.B, *fixed);
    else
      ASAP_LAUNCH(tm, "k_score_select", k_score_select, dim3(p.B), dim3(SEL_THREADS), lds, st, upart, s64, mmkey,
                  text_len, p.H, u_rows, p.V, p.k, p.Tmax, last_only, (double)p.lambda_max, (double)p.eps,
                  mask_on, s_hat, score, kept, pruned);
  } else {
    ASAP_LAUNCH(tm, "k_score", k_score, dim3((p.V + 63) / 64, p.B), dim3(256), 0, st, upart, s64, mmkey, text_len,
                p.H, u_rows, p.V, p.Tmax, last_only, (double)p.lambda_max, (double)p.eps, mask_on, s_hat, score);
  }
  return hipGetLastError();
}

hipError_t launch_score(const asap_params& p, const void* q_vis, Strides3 qv, const void* q_txt, Strides3 qt,
                        const void* k_vis, Strides3 kv, const int32_t* text_len, const float* lse_extra,
                        float* s_raw, float* s_hat, float* score, int32_t* kept, int32_t* pruned,
                        const FrontArgs* fe, const KvFixedRows* fixed, char* ws, size_t ws_budget, hipStream_t st,
                        Timer* tm) {
  if (fixed && (kept == nullptr || !score_fuses_selection(p))) return hipErrorInvalidValue;
  if (p.qk_dtype == ASAP_BF16)
    return score_typed<bf16_t>(p, q_vis, qv, q_txt, qt, k_vis, kv, text_len, lse_extra, s_raw, s_hat, score,
                               kept, pruned, fe, fixed, ws, ws_budget, st, tm);
  return score_typed<float>(p, q_vis, qv, q_txt, qt, k_vis, kv, text_len, lse_extra, s_raw, s_hat, score, kept,
                            pruned, fe, fixed, ws, ws_budget, st, tm);
}

}  // namespace asap
