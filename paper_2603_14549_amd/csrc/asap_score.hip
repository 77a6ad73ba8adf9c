// asap_score: Eq. 2 (raw attention mass), Eq. 3 (salience), Eq. 4 (discount) and the text-row
// softmax of Eq. 5 reduced to one selection score per visual token.
//
// Kernels, in launch order:
//   k_qsum        column sums of the visual queries per (image, head[, row chunk]); rows are added
//                 eight at a time in fp32, the eights in fp64
//   k_qsplit      fixed-order sum of those partials per kv head (fp64), also split into four bf16
//                 pieces per component (32 significant bits) for the matrix-core form of k_mass
//   k_mass        s_j = sum_g qbar_g . k_{g,j} / (H sqrt d)  (Eq. 2 by linearity) and the per-image
//                 min / max of s through order-preserving integer atomics.  bf16 keys: the four
//                 pieces of qbar are four query rows of an MFMA tile, products are exact, one head's
//                 128 products are added in fp32 and everything above that in fp64.  f32 keys: fp64
//                 FMAs on the vector ALUs.
//   k_attn_stats  per (image, head, key split): key x text-query logits on the matrix cores (keys as
//                 tile rows, so a lane owns one text row), online (max, sum) of lambda'_j 2^z per row
//   k_attn_colsum the sweep again with queries as tile rows and the merged row statistics:
//                 normalised column sums per key
//   k_score       fixed-order head reduction, times lambda' (Eq. 4) in fp64, mean over heads and
//                 text rows; also writes s_hat (Eq. 3)
//   k_score_select  the same followed by the top-k selection of asap_select in one launch (one
//                 workgroup per image), when the stage runs as one call
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
                         int H, int Hkv, int nchunk, int d) {
  const int g = blockIdx.x, b = blockIdx.y, c = threadIdx.x;
  const int G = H / Hkv;
  double s = 0.0;
  for (int h = g * G; h < (g + 1) * G; ++h)
    for (int ch = 0; ch < nchunk; ++ch) s += qpart[(((int64_t)b * H + h) * nchunk + ch) * d + c];
  qbar[((int64_t)b * Hkv + g) * d + c] = s;
  split_bf16x4(s, qsplit + ((int64_t)b * Hkv + g) * 4 * d + c, d);
}

// ------------------------------------------------------------------------------------------
// k_mass (vector-ALU form, f32 keys): grid (ceil(V/32), B), 256 threads, dynamic LDS = Hkv*d doubles
// (qbar of the image, stored so that lanes with consecutive pieces read consecutive 16 bytes).
// ------------------------------------------------------------------------------------------
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

template <typename T>
__global__ __launch_bounds__(256) void k_mass(const T* __restrict__ kv, Strides3 sk, const double* __restrict__ qbar,
                                               int Hkv, int V, int d, double scale, double* __restrict__ s64,
                                               float* __restrict__ s_raw, unsigned long long* __restrict__ mmkey) {
  constexpr int E = elem<T>::per16;
  constexpr int JT = 32;
  extern __shared__ __align__(16) double qb_s[];
  __shared__ unsigned long long blk_mm[2];
  const int LPR = d / E, RPI = 256 / LPR, NP = JT / RPI;   // NP passes of RPI rows
  const int tid = threadIdx.x, piece = tid % LPR, r0 = tid / LPR;
  const int b = blockIdx.y, j0 = blockIdx.x * JT;
  // qb_s[g][e / 2][piece][e % 2]: element e of piece `piece`
  for (int i = tid; i < Hkv * d; i += 256) {
    int g = i / d, col = i % d, pc = col / E, e = col % E;
    qb_s[g * d + (e >> 1) * (LPR * 2) + pc * 2 + (e & 1)] = qbar[(int64_t)b * Hkv * d + i];
  }
  if (tid == 0) { blk_mm[0] = ~0ull; blk_mm[1] = 0ull; }
  __syncthreads();
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  const char* base = reinterpret_cast<const char*>(kv + b * sk.b + piece * E);
  const int64_t rowb = sk.r * (int64_t)sizeof(T), headb = sk.h * (int64_t)sizeof(T);
  int rows[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) rows[p] = min(j0 + p * RPI + r0, V - 1);
  constexpr int GU = 4;                                // kv heads in flight
  for (int g0 = 0; g0 < Hkv; g0 += GU) {
    uint4 ch[GU][4];
#pragma unroll
    for (int u = 0; u < GU; ++u)
#pragma unroll
      for (int p = 0; p < 4; ++p)
        if (p < NP && g0 + u < Hkv) ch[u][p] = ldg16(base + (g0 + u) * headb + rows[p] * rowb);
#pragma unroll
    for (int u = 0; u < GU; ++u) {
      if (g0 + u < Hkv) {
        double qb[E];
        const double* qs = qb_s + (g0 + u) * d + piece * 2;
#pragma unroll
        for (int e = 0; e < E; e += 2) {
          double2 t2 = *reinterpret_cast<const double2*>(qs + (e >> 1) * (LPR * 2));
          qb[e] = t2.x;
          qb[e + 1] = t2.y;
        }
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          if (p < NP) {
            float f[E];
            unpack16<T>(ch[u][p], f);
#pragma unroll
            for (int e = 0; e < E; ++e) acc[p] = fma(qb[e], (double)f[e], acc[p]);
          }
        }
      }
    }
  }
  unsigned long long kmin = ~0ull, kmax = 0ull;
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
        unsigned long long key = f64_key(s);
        kmin = key < kmin ? key : kmin;
        kmax = key > kmax ? key : kmax;
      }
    }
  }
  publish_minmax(kmin, kmax, piece == 0, blk_mm, mmkey, b);
}

// One key of a 32-key tile per lane pair in the matrix-core operand layout: lane (n, hf) takes the
// 16-byte pieces 2c + hf (c < CH) of key n.  CH = 16-byte chunks of a row per lane half (d = 16*CH).
template <int CH>
__device__ __forceinline__ void load_key_tile(uint4 (&kb)[CH], const char* krow) {
#pragma unroll
  for (int c = 0; c < CH; ++c) kb[c] = ldg16(krow + c * 32);
}

// ------------------------------------------------------------------------------------------
// k_mass_mfma (bf16 keys): grid (ceil(V/32), B), 256 threads = 4 waves.  A workgroup owns one
// 32-key tile; wave w walks the kv heads g = w, w + 4, ...  The four bf16 pieces of qbar_g are rows
// 0..3 of the MFMA A tile (rows 4..31 are zero), the keys are the B tile, so lane n (< 32) finds
// the four partial dot products of key n in its first four accumulator registers.
// The tile of a head is an isolated 8 KiB piece of memory, and reading such pieces in the operand
// pattern (32 rows x 32 bytes per instruction) was measured at 4.2 TB/s against 6.0 TB/s for whole
// rows.  So a wave reads whole rows (2 CH consecutive lanes per row) and turns the tile into the
// operand layout through an LDS buffer of its own -- written and read by the same wave, in order, so
// no barrier is involved.  CH = 16-byte chunks of a row per lane half (d = 16 CH).
// ------------------------------------------------------------------------------------------
template <int CH>
__global__ __launch_bounds__(256) void k_mass_mfma(const bf16_t* __restrict__ kv, Strides3 sk,
                                                    const uint16_t* __restrict__ qsplit, int Hkv, int V,
                                                    double scale, double* __restrict__ s64, float* __restrict__ s_raw,
                                                    unsigned long long* __restrict__ mmkey) {
  constexpr int D = CH * 16, RB = 32 * CH;          // row bytes
  constexpr int LPR = 2 * CH, RPI = 64 / LPR;        // lanes per row, rows per load instruction
  __shared__ __align__(16) char stage[4][32 * RB];
  __shared__ double part[4][32];
  __shared__ unsigned long long blk_mm[2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, hf = lane >> 5;
  const int piece = lane % LPR, r0 = lane / LPR;
  const int b = blockIdx.y, j0 = blockIdx.x * 32;
  if (tid == 0) { blk_mm[0] = ~0ull; blk_mm[1] = 0ull; }
  const int64_t headb = sk.h * 2;
  // LDS: the 16-byte piece p of row r sits in slot p ^ x(r): whole-row writes and operand reads of 16
  // consecutive rows both cover all banks
  auto swz = [](int row) { return RB <= 128 ? (row >> 1) & 7 : row & 15; };
  char* st = stage[wave];
  uint32_t roff[CH];          // byte offsets inside one head of one image (< 4 GiB)
  int wr[CH];
#pragma unroll
  for (int i = 0; i < CH; ++i) {
    const int row = r0 + RPI * i;
    roff[i] = (uint32_t)(min(j0 + row, V - 1) * (int)sk.r * 2 + piece * 16);
    wr[i] = row * RB + ((piece ^ swz(row)) << 4);
  }
  // operand read c: piece (2c + hf) ^ x(n) of row n = rd0 ^ 32 c (the row offset has no low bits set)
  const int rd0 = n * RB + ((hf ^ swz(n)) << 4);
  const char* kbase = reinterpret_cast<const char*>(kv + b * sk.b);
  // lane (m, hf) with m < 4 supplies piece m of qbar_g, half hf of the components
  const char* qbase = reinterpret_cast<const char*>(qsplit + ((int64_t)b * Hkv * 4 + (n & 3)) * D) + hf * 16;
  const int64_t qheadb = (int64_t)4 * D * 2;
  const bool has_q = n < 4;
  uint4 qa[CH], kb[CH], kn[CH];
#pragma unroll
  for (int c = 0; c < CH; ++c) qa[c] = make_uint4(0, 0, 0, 0);
  int g = wave;
  if (g < Hkv) {
#pragma unroll
    for (int i = 0; i < CH; ++i) kb[i] = ldg16(kbase + g * headb + roff[i]);
    if (has_q) load_key_tile<CH>(qa, qbase + g * qheadb);
  }
  double sum = 0.0;
  for (; g < Hkv; g += 4) {
    const int gn = g + 4;
    if (gn < Hkv) {
#pragma unroll
      for (int i = 0; i < CH; ++i) kn[i] = ldg16(kbase + gn * headb + roff[i]);
    }
#pragma unroll
    for (int i = 0; i < CH; ++i) *reinterpret_cast<uint4*>(st + wr[i]) = kb[i];
    f32x16_t acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
    for (int c = 0; c < CH; ++c) mma32<bf16_t>(acc, qa[c], *reinterpret_cast<const uint4*>(st + (rd0 ^ (32 * c))));
    sum += ((double)acc[0] + (double)acc[1]) + ((double)acc[2] + (double)acc[3]);   // rows 0..3 (lanes < 32)
    if (gn < Hkv) {
      if (has_q) load_key_tile<CH>(qa, qbase + gn * qheadb);      // small, cached: not worth registers of its own
#pragma unroll
      for (int i = 0; i < CH; ++i) kb[i] = kn[i];
    }
  }
  if (hf == 0) part[wave][n] = sum;
  __syncthreads();
  unsigned long long kmin = ~0ull, kmax = 0ull;
  const int j = j0 + n;
  if (tid < 32 && j < V) {
    const double s = (((part[0][n] + part[1][n]) + part[2][n]) + part[3][n]) * scale;
    s64[(int64_t)b * V + j] = s;
    s_raw[(int64_t)b * V + j] = (float)s;
    kmin = kmax = f64_key(s);
  }
  publish_minmax(kmin, kmax, tid < 32, blk_mm, mmkey, b);
}

// ------------------------------------------------------------------------------------------
// Text-row attention sweeps.  grid (S, H, B), 256 threads = 4 waves.
//   RB = 32-row blocks of text queries (Tmax <= 32*RB); CH = 16-byte chunks of a row per lane half
//   (row bytes = 32*CH); QREG: the queries stay in registers as MFMA operands (else in LDS).
// Every wave streams its own 32-key tiles of the split's key range straight from global memory:
// lane (n, hf) of a tile reads the 16-byte pieces 2c + hf (c < CH) of key n -- the two lanes of a key
// take 32 contiguous bytes per load, which halves the cache lines a load instruction touches -- and
// the query side holds the same pieces of its row, so a chunk pair covers the same contraction slice.
// ------------------------------------------------------------------------------------------
struct AttnArgs {
  const void* qt; Strides3 sq;          // [B,H,Tmax,d]
  const void* kv; Strides3 sk;          // [B,Hkv,V,d]
  const double* s64;                    // [B,V]
  const unsigned long long* mmkey;      // [B,2]
  const int32_t* text_len;              // [B]
  const float* lse_extra;               // [B,H,Tmax] or null
  float* pstat;                         // [B,H,S,2,NR]   partial (max, sum) per text row
  float* upart;                         // [B,H,V]
  int H, Hkv, V, Tmax, S, tiles_per_split;
  float c2;                             // log2(e) / sqrt(d): accumulator units -> log2 units
  double lambda_max, eps;
  int mask_on;
};

// Query operands: registers or LDS.
template <typename T, int RB, int CH, bool QREG> struct QueryOps;
template <typename T, int RB, int CH> struct QueryOps<T, RB, CH, true> {
  uint4 qa[RB][CH];
  // rows at or past `len` (padding of a ragged batch, whatever it holds) become zero operands
  __device__ __forceinline__ void init(const AttnArgs& a, int b, int h, int lane, char*, int len) {
    const int m = lane & 31, hf = lane >> 5;
    const char* qbase = reinterpret_cast<const char*>(static_cast<const T*>(a.qt) + b * a.sq.b + h * a.sq.h) +
                        hf * 16;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const int row = rb * 32 + m;
#pragma unroll
      for (int c = 0; c < CH; ++c)
        qa[rb][c] = row < len ? ldg16(qbase + (int64_t)row * a.sq.r * sizeof(T) + c * 32) : make_uint4(0, 0, 0, 0);
    }
  }
  __device__ __forceinline__ uint4 get(int rb, int c) const { return qa[rb][c]; }
  static constexpr size_t lds_bytes() { return 0; }
};
template <typename T, int RB, int CH> struct QueryOps<T, RB, CH, false> {
  static constexpr int ROWB = CH * 32, LDSROW = ROWB + 16;
  const char* qa;
  __device__ __forceinline__ void init(const AttnArgs& a, int b, int h, int lane, char* lds, int len) {
    const char* qbase = reinterpret_cast<const char*>(static_cast<const T*>(a.qt) + b * a.sq.b + h * a.sq.h);
    constexpr int PPR = ROWB / 16;
    for (int i = threadIdx.x; i < RB * 32 * PPR; i += 256) {
      int row = i / PPR, pc = i % PPR;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (row < len) v = ldg16(qbase + (int64_t)row * a.sq.r * sizeof(T) + pc * 16);
      *reinterpret_cast<uint4*>(lds + row * LDSROW + pc * 16) = v;
    }
    __syncthreads();
    qa = lds + (lane & 31) * LDSROW + (lane >> 5) * 16;
  }
  __device__ __forceinline__ uint4 get(int rb, int c) const {
    return *reinterpret_cast<const uint4*>(qa + rb * 32 * LDSROW + c * 32);
  }
  static constexpr size_t lds_bytes() { return (size_t)RB * 32 * LDSROW; }
};

__device__ __forceinline__ float discount(const AttnArgs& a, int b, int j, double lo, double inv) {
  if (!a.mask_on) return 1.0f;
  return (float)fmax(a.lambda_max * ((a.s64[(int64_t)b * a.V + j] - lo) * inv), a.eps);
}

// merge of two (max, sum) pairs kept in accumulator units with scale c2
__device__ __forceinline__ void merge_stat(float& m, float& s, float m2, float s2, float c2) {
  float M = fmaxf(m, m2);
  s = s * fast_exp2((m - M) * c2) + s2 * fast_exp2((m2 - M) * c2);
  m = M;
}

// Keys are the tile rows here: lane (n, hf) owns text row rb*32 + n and finds, in accumulator
// register v, its logit against key 8*(v/4) + 4*hf + v%4 of the tile.
template <typename T, int RB, int CH, bool QREG>
__global__ __launch_bounds__(256, ((RB <= 2 && CH <= 8) ? 2 : 1)) void k_attn_stats(AttnArgs a) {
  constexpr int NR = RB * 32;
  constexpr bool PREF = CH * RB <= 32;     // next key tile prefetched into a second register set
  constexpr float NEG = -1e30f;
  extern __shared__ __align__(16) char lds[];
  using Q = QueryOps<T, RB, CH, QREG>;
  float* st_m = reinterpret_cast<float*>(lds + Q::lds_bytes());   // [4][NR]
  float* st_s = st_m + 4 * NR;                                     // [4][NR]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, hf = lane >> 5;
  const int sp = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int g = (h * a.Hkv) / a.H;
  const int len = min(max(a.text_len[b], 0), a.Tmax);
  const int nrb = (len + 31) >> 5;          // row blocks that hold a valid text row of this image
  Q q;
  q.init(a, b, h, lane, lds, len);
  const double mlo = f64_unkey(a.mmkey[2 * b]), mhi = f64_unkey(a.mmkey[2 * b + 1]);
  const double minv = 1.0 / (mhi - mlo + a.eps);
  const char* kbase = reinterpret_cast<const char*>(static_cast<const T*>(a.kv) + b * a.sk.b + g * a.sk.h) +
                      hf * 16;
  const int64_t krow_bytes = a.sk.r * (int64_t)sizeof(T);
  const int ntiles = (a.V + 31) >> 5;
  const int t_end = min(ntiles, (sp + 1) * a.tiles_per_split);
  const float c2 = a.c2;

  float m_run[RB], s_run[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) { m_run[rb] = NEG; s_run[rb] = 0.0f; }

  uint4 kb[CH], kn[CH];
  int tile = sp * a.tiles_per_split + wave;
  if (tile < t_end) load_key_tile<CH>(kb, kbase + (int64_t)min(tile * 32 + n, a.V - 1) * krow_bytes);
  for (; tile < t_end; tile += 4) {
    const int j = tile * 32 + n;
    const int tnext = tile + 4;
    if (PREF && tnext < t_end) load_key_tile<CH>(kn, kbase + (int64_t)min(tnext * 32 + n, a.V - 1) * krow_bytes);
    // discount of key n of the tile, then handed to the lanes in accumulator order
    const float lj = j < a.V ? discount(a, b, j, mlo, minv) : 0.0f;
    float lam[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) lam[v] = __shfl(lj, 8 * (v >> 2) + 4 * hf + (v & 3));
    const bool ragged = tile * 32 + 32 > a.V;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      if (rb >= nrb) continue;               // wave-uniform: nothing but padding in this block
      f32x16_t acc;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
      for (int c = 0; c < CH; ++c) mma32<T>(acc, kb[c], q.get(rb, c));
      if (ragged) {
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (tile * 32 + 8 * (v >> 2) + 4 * hf + (v & 3) >= a.V) acc[v] = NEG;
      }
      float mx = acc[0];
#pragma unroll
      for (int v = 1; v < 16; ++v) mx = fmaxf(mx, acc[v]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));                  // both halves of the row's 32 keys
      const float m_new = fmaxf(m_run[rb], mx);
      float s = s_run[rb] * fast_exp2((m_run[rb] - m_new) * c2);
      const float off = -m_new * c2;
#pragma unroll
      for (int v = 0; v < 16; ++v) s = fmaf(lam[v], fast_exp2(fmaf(acc[v], c2, off)), s);
      s_run[rb] = s;
      m_run[rb] = m_new;
    }
    if (tnext < t_end) {
      if (PREF) {
#pragma unroll
        for (int c = 0; c < CH; ++c) kb[c] = kn[c];
      } else {
        load_key_tile<CH>(kb, kbase + (int64_t)min(tnext * 32 + n, a.V - 1) * krow_bytes);
      }
    }
  }
  // the two halves of a wave share the row maximum: their sums just add; then the 4 waves
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float s = s_run[rb] + __shfl_xor(s_run[rb], 32);
    if (hf == 0) {
      st_m[wave * NR + rb * 32 + n] = m_run[rb];
      st_s[wave * NR + rb * 32 + n] = s;
    }
  }
  __syncthreads();
  if (tid < NR) {
    float m = st_m[tid], s = st_s[tid];
    for (int w = 1; w < 4; ++w) merge_stat(m, s, st_m[w * NR + tid], st_s[w * NR + tid], c2);
    float* out = a.pstat + ((((int64_t)b * a.H + h) * a.S + sp) * 2) * NR;
    out[tid] = m;
    out[NR + tid] = s;
  }
}

// Queries are the tile rows here: lane (n, hf) owns key n of the tile and finds, in accumulator
// register v of row block rb, its logit against text row rb*32 + 8*(v/4) + 4*hf + v%4.
template <typename T, int RB, int CH, bool QREG>
__global__ __launch_bounds__(256, ((RB <= 2 && CH <= 8) ? 2 : 1)) void k_attn_colsum(AttnArgs a) {
  constexpr int NR = RB * 32;
  constexpr bool PREF = CH * RB <= 32;
  extern __shared__ __align__(16) char lds[];
  using Q = QueryOps<T, RB, CH, QREG>;
  float* fin_o = reinterpret_cast<float*>(lds + Q::lds_bytes());   // [NR]  -max * c2
  float* fin_i = fin_o + NR;                                       // [NR]  1 / denominator
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, hf = lane >> 5;
  const int sp = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int g = (h * a.Hkv) / a.H;
  const int len = min(max(a.text_len[b], 0), a.Tmax);
  const int nrb = (len + 31) >> 5;
  const float c2 = a.c2;
  // merged row statistics of this (image, head): fixed order over the splits
  if (tid < NR) {
    const float* ps = a.pstat + (((int64_t)b * a.H + h) * a.S * 2) * NR;
    float m = ps[tid], s = ps[NR + tid];
    for (int w = 1; w < a.S; ++w) merge_stat(m, s, ps[(w * 2) * NR + tid], ps[(w * 2 + 1) * NR + tid], c2);
    float m2 = m * c2;                                             // log2 units from here on
    if (a.lse_extra != nullptr && tid < a.Tmax) {
      float l2 = a.lse_extra[((int64_t)b * a.H + h) * a.Tmax + tid] * 1.4426950408889634f;
      float M = fmaxf(m2, l2);
      s = s * fast_exp2(m2 - M) + fast_exp2(l2 - M);
      m2 = M;
    }
    const bool row_ok = tid < len;
    fin_o[tid] = row_ok ? -m2 : -INFINITY;   // 2^(z - inf) = 0: padded rows add nothing
    fin_i[tid] = row_ok ? 1.0f / s : 0.0f;
  }
  Q q;
  q.init(a, b, h, lane, lds, len);
  __syncthreads();
  float off[RB][16], inv[RB][16];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      int row = rb * 32 + mma32_row(v, lane);
      off[rb][v] = fin_o[row];
      inv[rb][v] = fin_i[row];
    }
  const char* kbase = reinterpret_cast<const char*>(static_cast<const T*>(a.kv) + b * a.sk.b + g * a.sk.h) +
                      hf * 16;
  const int64_t krow_bytes = a.sk.r * (int64_t)sizeof(T);
  const int ntiles = (a.V + 31) >> 5;
  const int t_end = min(ntiles, (sp + 1) * a.tiles_per_split);
  float* out = a.upart + ((int64_t)b * a.H + h) * a.V;
  uint4 kb[CH], kn[CH];
  int tile = sp * a.tiles_per_split + wave;
  if (tile < t_end) load_key_tile<CH>(kb, kbase + (int64_t)min(tile * 32 + n, a.V - 1) * krow_bytes);
  for (; tile < t_end; tile += 4) {
    const int j = tile * 32 + n;
    const int tnext = tile + 4;
    if (PREF && tnext < t_end) load_key_tile<CH>(kn, kbase + (int64_t)min(tnext * 32 + n, a.V - 1) * krow_bytes);
    float u = 0.0f;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      if (rb >= nrb) continue;               // wave-uniform: padded rows add nothing
      f32x16_t acc;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
      for (int c = 0; c < CH; ++c) mma32<T>(acc, q.get(rb, c), kb[c]);
#pragma unroll
      for (int v = 0; v < 16; ++v) u = fmaf(fast_exp2(fmaf(acc[v], c2, off[rb][v])), inv[rb][v], u);
    }
    u += __shfl_xor(u, 32);
    if (hf == 0 && j < a.V) out[j] = u;
    if (tnext < t_end) {
      if (PREF) {
#pragma unroll
        for (int c = 0; c < CH; ++c) kb[c] = kn[c];
      } else {
        load_key_tile<CH>(kb, kbase + (int64_t)min(tnext * 32 + n, a.V - 1) * krow_bytes);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// k_score: grid (ceil(V/64), B), 256 threads: 64 keys x 4 head groups.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_score(const float* __restrict__ upart, const double* __restrict__ s64,
                                                const unsigned long long* __restrict__ mmkey,
                                                const int32_t* __restrict__ text_len, int H, int V,
                                                double lambda_max, double eps, int mask_on,
                                                float* __restrict__ s_hat, float* __restrict__ score) {
  __shared__ double part[4][64];
  const int b = blockIdx.y, jl = threadIdx.x & 63, hq = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + jl;
  double u = 0.0;
  if (j < V) {
    const float* up = upart + (int64_t)b * H * V + j;
    int h = hq;
    for (; h + 12 < H; h += 16) {
      float u0 = up[(int64_t)h * V], u1 = up[(int64_t)(h + 4) * V], u2 = up[(int64_t)(h + 8) * V],
            u3 = up[(int64_t)(h + 12) * V];
      u += (double)u0;
      u += (double)u1;
      u += (double)u2;
      u += (double)u3;
    }
    for (; h < H; h += 4) u += (double)up[(int64_t)h * V];
  }
  part[hq][jl] = u;
  __syncthreads();
  if (hq == 0 && j < V) {
    u = ((part[0][jl] + part[1][jl]) + part[2][jl]) + part[3][jl];
    const double lo = f64_unkey(mmkey[2 * b]), hi = f64_unkey(mmkey[2 * b + 1]);
    const double sh = (s64[(int64_t)b * V + j] - lo) * (1.0 / (hi - lo + eps));
    const double lam = mask_on ? fmax(lambda_max * sh, eps) : 1.0;
    s_hat[(int64_t)b * V + j] = (float)sh;
    score[(int64_t)b * V + j] = (float)(lam * u / ((double)H * (double)text_len[b]));
  }
}

// ------------------------------------------------------------------------------------------
// k_score_select: grid (B), 1024 threads.  Thread t owns the keys t*ipt .. t*ipt+ipt-1 of its image:
// it reduces their per-head column sums in the order k_score uses (four interleaved head groups in
// fp64, then ((0+1)+2)+3), so that score and s_hat come out bit-identical to k_score's, and the
// workgroup then selects exactly as k_select does.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(SEL_THREADS) void k_score_select(const float* __restrict__ upart,
                                                               const double* __restrict__ s64,
                                                               const unsigned long long* __restrict__ mmkey,
                                                               const int32_t* __restrict__ text_len, int H, int V,
                                                               int k, double lambda_max, double eps, int mask_on,
                                                               float* __restrict__ s_hat, float* __restrict__ score,
                                                               int32_t* __restrict__ kept,
                                                               int32_t* __restrict__ pruned) {
  __shared__ SelectShared sh;
  const int b = blockIdx.x, tid = threadIdx.x;
  const int ipt = (V + SEL_THREADS - 1) / SEL_THREADS;
  const int i0 = tid * ipt;
  const double lo = f64_unkey(mmkey[2 * b]), hi = f64_unkey(mmkey[2 * b + 1]);
  const double inv = 1.0 / (hi - lo + eps);
  const double norm = (double)H * (double)text_len[b];
  const float* up = upart + (int64_t)b * H * V;
  uint32_t key[SEL_IPT];
#pragma unroll
  for (int e = 0; e < SEL_IPT; ++e) {
    const int j = i0 + e;
    key[e] = 0u;
    if (e < ipt && j < V) {
      double part[4] = {0.0, 0.0, 0.0, 0.0};
      int h = 0;
      for (; h + 16 <= H; h += 16) {          // 16 loads in flight; head h adds to group h % 4, in order
        float u[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) u[q] = up[(int64_t)(h + q) * V + j];
#pragma unroll
        for (int q = 0; q < 16; ++q) part[q & 3] += (double)u[q];
      }
      for (; h < H; ++h) part[h & 3] += (double)up[(int64_t)h * V + j];
      const double usum = ((part[0] + part[1]) + part[2]) + part[3];
      const double shat = (s64[(int64_t)b * V + j] - lo) * inv;
      const double lam = mask_on ? fmax(lambda_max * shat, eps) : 1.0;
      const float sc = (float)(lam * usum / norm);
      s_hat[(int64_t)b * V + j] = (float)shat;
      score[(int64_t)b * V + j] = sc;
      key[e] = float_key(sc);
    }
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

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
// Key-range splits of the two text-row sweeps.  Their workgroups run in rounds of as many as fit
// on the chip at once (1 to 4 per compute unit, by the registers of the instantiation); a round
// costs the tiles of one split plus a fixed part (start-up, the text queries, the last tiles' tail:
// about 8 tile times, fitted to measurements), and more than one workgroup per compute unit at a
// time slows each of them (about 1.4x).  The count with the least modelled time wins, fewer splits
// on ties; a split has at least 4 tiles (one per wave).
static int attn_splits(const asap_params& p) {
  const int ntiles = (p.V + 31) / 32;
  const int rb = (p.Tmax + 31) / 32, ch = p.d / (p.qk_dtype == ASAP_BF16 ? 16 : 8);
  const int per_cu = rb * ch <= 4 ? 4 : (rb * ch <= 8 && ch == 8) ? 3 : (rb * ch <= 16 && ch <= 8) ? 2 : 1;
  const long slots = 256L * per_cu, groups = (long)p.H * p.B;
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

ScoreWorkspace score_workspace(const asap_params& p) {
  ScoreWorkspace w;
  // rows per k_qsum block: whole image span unless that leaves the chip short of blocks
  int chunks = (512 + p.B * p.H - 1) / (p.B * p.H);
  if (chunks > (p.V + 255) / 256) chunks = (p.V + 255) / 256;
  if (chunks < 1) chunks = 1;
  w.q_rows = (p.V + chunks - 1) / chunks;
  w.q_chunks = (p.V + w.q_rows - 1) / w.q_rows;
  w.attn_splits = attn_splits(p);
  const int NR = ((p.Tmax + 31) / 32) * 32;
  size_t off = 0;
  w.off_qpart = off;  off = align256(off + sizeof(double) * p.B * p.H * w.q_chunks * p.d);
  w.off_qbar = off;   off = align256(off + sizeof(double) * p.B * p.Hkv * p.d);
  w.off_qsplit = off; off = align256(off + sizeof(uint16_t) * p.B * p.Hkv * 4 * p.d);
  w.off_s64 = off;    off = align256(off + sizeof(double) * p.B * p.V);
  w.off_mm = off;     off = align256(off + sizeof(double) * p.B * 2);
  w.off_pstat = off;  off = align256(off + sizeof(float) * (size_t)p.B * p.H * w.attn_splits * 2 * NR);
  w.off_upart = off;  off = align256(off + sizeof(float) * (size_t)p.B * p.H * p.V);
  w.total = off;
  return w;
}

template <typename T, int RB, int CH, bool QREG>
static hipError_t launch_attn(const asap_params& p, const AttnArgs& a, hipStream_t st, Timer* tm) {
  constexpr int NR = RB * 32;
  using Q = QueryOps<T, RB, CH, QREG>;
  const size_t lds = Q::lds_bytes() + sizeof(float) * 8 * NR;
  auto k1 = k_attn_stats<T, RB, CH, QREG>;
  auto k2 = k_attn_colsum<T, RB, CH, QREG>;
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k1),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(k2), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)lds);
    if (e != hipSuccess) return e;
  }
  ASAP_LAUNCH(tm, "k_attn_stats", k1, dim3(a.S, p.H, p.B), dim3(256), lds, st, a);
  ASAP_LAUNCH(tm, "k_attn_colsum", k2, dim3(a.S, p.H, p.B), dim3(256), lds, st, a);
  return hipGetLastError();
}

template <typename T, int CH>
static hipError_t dispatch_rb(const asap_params& p, const AttnArgs& a, hipStream_t st, Timer* tm) {
  // queries stay in registers while they need at most 64 VGPRs
  constexpr bool R1 = CH * 4 <= 64, R2 = CH * 8 <= 64;
  switch ((p.Tmax + 31) / 32) {
    case 1: return launch_attn<T, 1, CH, R1>(p, a, st, tm);
    case 2: return launch_attn<T, 2, CH, R2>(p, a, st, tm);
    case 3: return launch_attn<T, 3, CH, false>(p, a, st, tm);
    case 4: return launch_attn<T, 4, CH, false>(p, a, st, tm);
  }
  return hipErrorInvalidValue;
}

template <typename T>
static hipError_t score_typed(const asap_params& p, const void* q_vis, Strides3 qv, const void* q_txt,
                              Strides3 qt, const void* k_vis, Strides3 kv, const int32_t* text_len,
                              const float* lse_extra, float* s_raw, float* s_hat, float* score, int32_t* kept,
                              int32_t* pruned, char* ws, hipStream_t st, Timer* tm) {
  const ScoreWorkspace w = score_workspace(p);
  double* qpart = reinterpret_cast<double*>(ws + w.off_qpart);
  double* qbar = reinterpret_cast<double*>(ws + w.off_qbar);
  uint16_t* qsplit = reinterpret_cast<uint16_t*>(ws + w.off_qsplit);
  double* s64 = reinterpret_cast<double*>(ws + w.off_s64);
  unsigned long long* mmkey = reinterpret_cast<unsigned long long*>(ws + w.off_mm);
  float* pstat = reinterpret_cast<float*>(ws + w.off_pstat);
  float* upart = reinterpret_cast<float*>(ws + w.off_upart);
  const int mask_on = p.mask_mode == ASAP_MASK_KEYBIAS;
  constexpr int E = elem<T>::per16;
  const int ch = p.d / E / 2;   // 16-byte chunks per half row
  const int ktiles = (p.V + 31) / 32;

  const int direct = (w.q_chunks == 1 && p.H == p.Hkv) ? 1 : 0;
  ASAP_LAUNCH(tm, "k_qsum", k_qsum<T>, dim3(w.q_chunks, p.H, p.B), dim3(1024), 0, st, static_cast<const T*>(q_vis),
              qv, p.V, p.d, w.q_rows, qpart, mmkey, qbar, qsplit, direct);
  if (!direct)
    ASAP_LAUNCH(tm, "k_qsplit", k_qsplit, dim3(p.Hkv, p.B), dim3(p.d), 0, st, qpart, qbar, qsplit, p.H, p.Hkv,
                w.q_chunks, p.d);
  const double scale = 1.0 / ((double)p.H * sqrt((double)p.d));
  if constexpr (E == 8) {
    const bf16_t* kp = static_cast<const bf16_t*>(k_vis);
    if (ch == 8)
      ASAP_LAUNCH(tm, "k_mass", k_mass_mfma<8>, dim3(ktiles, p.B), dim3(256), 0, st, kp, kv, qsplit, p.Hkv, p.V, scale,
                  s64, s_raw, mmkey);
    else
      ASAP_LAUNCH(tm, "k_mass", k_mass_mfma<4>, dim3(ktiles, p.B), dim3(256), 0, st, kp, kv, qsplit, p.Hkv, p.V, scale,
                  s64, s_raw, mmkey);
  } else {
    ASAP_LAUNCH(tm, "k_mass", k_mass<T>, dim3(ktiles, p.B), dim3(256), sizeof(double) * p.Hkv * p.d, st,
                static_cast<const T*>(k_vis), kv, qbar, p.Hkv, p.V, p.d, scale, s64, s_raw, mmkey);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;

  AttnArgs a;
  a.qt = q_txt; a.sq = qt; a.kv = k_vis; a.sk = kv; a.s64 = s64; a.mmkey = mmkey; a.text_len = text_len;
  a.lse_extra = lse_extra; a.pstat = pstat; a.upart = upart;
  a.H = p.H; a.Hkv = p.Hkv; a.V = p.V; a.Tmax = p.Tmax; a.S = w.attn_splits;
  a.tiles_per_split = (ktiles + a.S - 1) / a.S;
  a.c2 = (float)(1.4426950408889634 / sqrt((double)p.d));
  a.lambda_max = (double)p.lambda_max; a.eps = (double)p.eps; a.mask_on = mask_on;
  if (ch == 4) {
    if constexpr (E == 8) e = dispatch_rb<T, 4>(p, a, st, tm);
    else e = hipErrorInvalidValue;
  } else if (ch == 8) {
    e = dispatch_rb<T, 8>(p, a, st, tm);
  } else if (ch == 16) {
    if constexpr (E == 4) e = dispatch_rb<T, 16>(p, a, st, tm);
    else e = hipErrorInvalidValue;
  } else {
    e = hipErrorInvalidValue;
  }
  if (e != hipSuccess) return e;
  if (kept != nullptr)
    ASAP_LAUNCH(tm, "k_score_select", k_score_select, dim3(p.B), dim3(SEL_THREADS), 0, st, upart, s64, mmkey,
                text_len, p.H, p.V, p.k, (double)p.lambda_max, (double)p.eps, mask_on, s_hat, score, kept, pruned);
  else
    ASAP_LAUNCH(tm, "k_score", k_score, dim3((p.V + 63) / 64, p.B), dim3(256), 0, st, upart, s64, mmkey, text_len,
                p.H, p.V, (double)p.lambda_max, (double)p.eps, mask_on, s_hat, score);
  return hipGetLastError();
}

hipError_t launch_score(const asap_params& p, const void* q_vis, Strides3 qv, const void* q_txt, Strides3 qt,
                        const void* k_vis, Strides3 kv, const int32_t* text_len, const float* lse_extra,
                        float* s_raw, float* s_hat, float* score, int32_t* kept, int32_t* pruned, char* ws,
                        hipStream_t st, Timer* tm) {
  if (p.qk_dtype == ASAP_BF16)
    return score_typed<bf16_t>(p, q_vis, qv, q_txt, qt, k_vis, kv, text_len, lse_extra, s_raw, s_hat, score,
                               kept, pruned, ws, st, tm);
  return score_typed<float>(p, q_vis, qv, q_txt, qt, k_vis, kv, text_len, lse_extra, s_raw, s_hat, score, kept,
                            pruned, ws, st, tm);
}

}  // namespace asap
