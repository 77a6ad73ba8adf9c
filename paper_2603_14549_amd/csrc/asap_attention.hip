// asap_attention: the attention forward of one decoder layer in front of the pruning layer under the
// salience-guided bidirectional mask (Eq. 4-5 on the whole sequence; Eq. 1 with the mask off):
//   out[b,h,i,:] = sum_j A_ij v[b,g(h),j,:],  A_i. = softmax_j( q_i.k_j / sqrt(d) + M_ij ),
//   M_ij = 0 (j <= i);  ln(max(lambda_max s_hat_j, eps)) (j > i, both inside the image span);  -inf otherwise.
// Flash-style: one pass over the keys with running row maxima and sums, both contractions on the
// matrix cores, nothing of size N x N ever stored.
//
//   k_att_bias      log2 of the per-key discount by sequence position, [B,Npad] (-inf off the image span,
//                   and everywhere with the mask off)
//   k_vtranspose    values transposed per (image, kv head) to [d, Npad]: the second contraction wants
//                   its A operand (a row of values^T) contiguous along the keys, in the key order in
//                   which the first contraction leaves P^T in the accumulators.  Not needed for bf16
//                   with d = 128: there the values go to LDS row-major and the operand is fetched
//                   with the chip's transposing LDS read (ds_read_b64_tr_b16), two per operand.
//   k_attention     grid (ceil(N/256), H, B), 512 threads = 8 waves (two per SIMD) of 32 queries.  Per
//                   32-key tile a wave computes S^T = K_tile Q^T (keys are the tile rows, so lane l owns
//                   query l % 32 and holds 16 of the tile's keys: the softmax bookkeeping is per lane),
//                   then O^T += V^T_tile P^T, where the P^T operand is taken straight from the
//                   accumulator registers: the contraction slice a lane half supplies is defined as
//                   the keys that lane half already holds, and the V^T operand is stored to match.
//                   A tile (keys, values^T, 32 discounts) goes to LDS by direct global -> LDS loads,
//                   once for the eight waves, into a ring of PD + 2 slots, PD tiles ahead; the waits
//                   for those loads are placed by hand and no other vector-memory instruction is left
//                   in the loop, because any wait the compiler adds for one would drain the ring.
//                   The raw scores of tile t + 1 are computed in the same basic block as the
//                   exponentials of tile t.  Measured on this chip, plain VALU work overlaps with the
//                   matrix pipe only up to about one VALU instruction per 8 MFMA cycles and SIMD, the
//                   rest adds to the MFMA time: the ~115 VALU instructions of a tile against its 16
//                   MFMAs are what bounds the kernel.
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
  if (s_hat != nullptr && j >= P && j < P + V) x = log2f(fmaxf(lambda_max * s_hat[(int64_t)b * V + (j - P)], eps));
  bias2[(int64_t)b * Npad + j] = x;
}

// grid (ceil(Npad/32), Hkv, B), 256 threads; vt[b,g,c,p] = v[b,g,att_vt_key(p),c] for keys < N, 0 for the
// keys N .. Npad-1.
// 16-byte loads along d into LDS, 16-byte stores along the keys out of it.
// Key stored at position p of a values^T row.  The second product takes its P^T operand straight from
// the accumulators of the first, where a lane half holds keys 4 hf .. 4 hf + 3 and 8 + 4 hf .. 8 + 4 hf + 3 of
// every 16; with 2-byte elements (8 keys per 16-byte operand) the row is therefore stored in the order
// 0-3, 8-11, 4-7, 12-15 within every 16 keys, so that a lane half's operand is one contiguous piece.
__device__ __forceinline__ int att_vt_key(int p, int elems_per_16) {
  if (elems_per_16 != 8) return p;
  const int g = p & 15;
  return (p & ~15) | (g & 3) | ((g & 4) << 1) | ((g & 8) >> 1);
}

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
    for (int e = 0; e < E; ++e) x[e] = tile[att_vt_key(r0 + e, E)][c];
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

// The transposing LDS read of gfx950 for 16-bit elements (ds_read_b64_tr_b16): every lane names 8
// bytes; in each group of 16 lanes, lane 4 a + c receives the c-th 16-bit element of the pieces named
// by lanes a, 4 + a, 8 + a and 12 + a, in that order.
typedef short att_i16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint2 att_tr_read(const char* lds_ptr) {
  const att_i16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) att_i16x4*)(uintptr_t)lds_address(lds_ptr));
  uint2 u;
  __builtin_memcpy(&u, &r, 8);
  return u;
}

// key held in accumulator register v of a lane of half hf, relative to the tile
__device__ __forceinline__ int att_key_of(int v, int hf) { return 8 * (v >> 2) + 4 * hf + (v & 3); }

constexpr int ATT_QWG = 256;                   // queries per workgroup
#ifndef ATT_PD
#define ATT_PD 2                               /* key tiles requested ahead */
#endif
constexpr int ATT_NW = 8;                      // waves per workgroup (two per SIMD), 32 queries each
constexpr float ATT_LAZY = 8.0f;               // growth of a row maximum (log2 units) that moves the baseline
constexpr int ATT_BIASB = 128;                 // bytes of per-key log-discounts staged with a key tile

// LDS swizzles: the 16-byte piece p of row r is stored in slot p ^ x(r), so that 16 consecutive rows
// spread over all banks for the strided operand reads while the loads still write 1 KiB at a time
__device__ __forceinline__ int att_kswz(int row, int row_bytes) { return row_bytes <= 128 ? (row >> 1) & 7 : row & 15; }
__device__ __forceinline__ int att_vswz(int row, int row_bytes) { return row_bytes <= 64 ? (row >> 2) & 3 : (row >> 1) & 7; }

// how the mask acts on one (32 keys x 32 queries) tile
enum { ATT_PLAIN = 0,     // every key precedes every query: no mask
       ATT_AHEAD = 1,     // every key follows every query and all queries are image rows: the key's discount
       ATT_GENERAL = 2 }; // anything else: decided per element

// wait until only the loads of the newest `tiles_ahead` key tiles (cnt instructions each) are outstanding
__device__ __forceinline__ void att_wait_tiles(int outstanding) {
  switch (outstanding) {
    case 0: wait_vmem_but<0>(); break;
    case 1: wait_vmem_but<1>(); break;
    case 2: wait_vmem_but<2>(); break;
    case 3: wait_vmem_but<3>(); break;
    case 4: wait_vmem_but<4>(); break;
    case 5: wait_vmem_but<5>(); break;
    case 6: wait_vmem_but<6>(); break;
    default: wait_vmem_but<0>(); break;
  }
}

// CH = 16-byte chunks of a row per lane half (row bytes = 32 * CH); PD = key tiles requested ahead
template <typename T, int CH, int PD>
__global__ __launch_bounds__(64 * ATT_NW) void k_attention(const T* __restrict__ q, Strides3 sq,
                                                            const T* __restrict__ k, Strides3 sk,
                                                            const T* __restrict__ vt, int Npad,
                                                            const T* __restrict__ vrm, Strides3 sv,
                                                            const float* __restrict__ bias2, int bidir,
                                                            T* __restrict__ out, int H, int Hkv, int N, int P, int V,
                                                            float c2) {
  constexpr int NW = ATT_NW;
  static_assert(NW * 32 == ATT_QWG, "workgroup shape");
  constexpr int E = elem<T>::per16;            // elements per 16-byte chunk
  constexpr int D = CH * 2 * E;                // head dimension
  constexpr int DT = D / 32;                   // 32-row tiles of O^T
  constexpr int NPS = 32 / (2 * E);            // contraction steps of the second product per key tile
  constexpr int RB = 32 * CH;                  // bytes of a key row
  constexpr int VB = 32 * (int)sizeof(T);      // bytes of a values^T row per key tile
  constexpr int KTILE = 32 * RB, VTILE = D * VB, STAGE = KTILE + VTILE + ATT_BIASB;
  constexpr int KLD = KTILE / 1024, VLD = VTILE / 1024;     // 1 KiB load instructions per tile
  constexpr int TP = KLD + VLD + 1;            // load instructions per tile: keys, values^T, discounts
  constexpr int NS = PD + 2;                   // ring slots: tile t (values, discounts), t+1 (keys), PD in flight
  // 2-byte elements with d = 128: the values stay row-major, as the caller has them, and the second
  // product's operand is fetched with the transposing LDS read of this chip (see att_tr_read)
  constexpr bool TR = (E == 8 && CH == 8);
  extern __shared__ __align__(16) char lds[];
  const uint32_t lds_addr = lds_address(lds);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, hf = lane >> 5;
  const int b = blockIdx.z, h = blockIdx.y, g = (h * Hkv) / H;
  const int iw = blockIdx.x * ATT_QWG;          // first query of the workgroup
  const int i0 = iw + wave * 32;                // first query of the wave
  const float inv_c2 = 1.0f / c2;
  const float lazy_raw = ATT_LAZY * inv_c2;     // ATT_LAZY log2 units, in units of the raw products
  const int img_lo = P, img_hi = P + V;         // image span [img_lo, img_hi)

  // keys to visit: up to the last query, or to the end of the image span if image rows are held
  // (their future image keys count, discounted)
  auto last_key = [&](int first, int count) {
    const int hi = min(first + count - 1, N - 1);
    int jl = hi;
    if (bidir && hi >= img_lo && first < img_hi) jl = max(jl, img_hi - 1);
    return first < N ? jl : -1;
  };
  const int jl_wg = last_key(iw, ATT_QWG), jl_w = last_key(i0, 32);
  const int ntiles = jl_wg / 32 + 1;
  const int my_tiles = jl_w / 32 + 1;           // this wave's tiles are 0 .. my_tiles-1 (none if its queries are past N)

  // queries: B operand of S^T, pieces 2c + hf of the row
  uint4 qa[CH];
  const int qi = i0 + n;
  {
    const char* qrow =
        reinterpret_cast<const char*>(q + b * sq.b + h * sq.h + (int64_t)min(qi, N - 1) * sq.r) + hf * 16;
#pragma unroll
    for (int c = 0; c < CH; ++c) qa[c] = ldg16(qrow + c * 32);
  }

  // Tile loads: the 1 KiB pieces of a tile (keys, then values^T, then one piece with the 32 discounts)
  // are dealt to the waves round-robin.  Tile numbers past the last one load the last tile again, so
  // every iteration issues the same number of loads and one wait count serves the whole loop.
  const char* kg = reinterpret_cast<const char*>(k + b * sk.b + g * sk.h);
  const int64_t krow_bytes = sk.r * (int64_t)sizeof(T);
  const char* vg = TR ? reinterpret_cast<const char*>(vrm + b * sv.b + g * sv.h)
                      : reinterpret_cast<const char*>(vt + ((int64_t)b * Hkv + g) * D * Npad);
  const int64_t vrow_bytes = sv.r * (int64_t)sizeof(T);
  const char* bg = reinterpret_cast<const char*>(bias2 + (int64_t)b * Npad);
  auto issue_tile = [&](auto slot_c, int t) {          // tile t goes to ring slot t % NS = slot_c
    const uint32_t st = lds_addr + (uint32_t)decltype(slot_c)::value * STAGE;
    const int j0 = min(t, ntiles - 1) * 32;
#pragma unroll
    for (int u = 0; u < (TP + NW - 1) / NW; ++u) {
      const int pc = wave + NW * u;
      if (pc < KLD) {
        const int off = pc * 1024 + 16 * lane, row = off / RB, slot = (off % RB) >> 4;
        const int piece = slot ^ att_kswz(row, RB);
        const uint32_t voff = (uint32_t)((int64_t)min(j0 + row, N - 1) * krow_bytes) + piece * 16;
        load_to_lds16(kg, voff, st + pc * 1024);
      } else if (pc < KLD + VLD) {
        const int pv = pc - KLD;
        if constexpr (TR) {
          // row-major values: 4 key rows of 256 bytes per instruction, piece p of row r in slot p ^ 4 (r & 3)
          const int off = pv * 1024 + 16 * lane, row = off / RB, slot = (off % RB) >> 4;
          const int piece = slot ^ ((row & 3) << 2);
          const uint32_t voff = (uint32_t)((int64_t)min(j0 + row, N - 1) * vrow_bytes) + piece * 16;
          load_to_lds16(vg, voff, st + KTILE + pv * 1024);
        } else {
          const int off = pv * 1024 + 16 * lane, row = off / VB, slot = (off % VB) >> 4;
          const int piece = slot ^ att_vswz(row, VB);
          const uint32_t voff = (uint32_t)(((int64_t)row * Npad + j0) * sizeof(T)) + piece * 16;
          load_to_lds16(vg, voff, st + KTILE + pv * 1024);
        }
      } else if (pc < TP) {
        if (lane < ATT_BIASB / 16) load_to_lds16(bg, (uint32_t)(j0 * 4 + 16 * lane), st + KTILE + VTILE);
      }
    }
  };
  const int my_loads = TP / NW + (wave < TP % NW ? 1 : 0);     // load instructions of this wave per tile

  f32x16_t o[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[t][v] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;

  // operand read offsets inside a tile.  The values^T swizzle of row tt * 32 + n does not depend on tt
  // (it looks at row bits below 5 only), so one offset per contraction step serves all DT row tiles.
  const int k_off = n * RB, k_x = att_kswz(n, RB);
  int v_off[NPS];
#pragma unroll
  for (int c = 0; c < NPS; ++c) v_off[c] = n * VB + (((2 * c + hf) ^ att_vswz(n, VB)) << 4);

  // Transposing read (TR): a lane is both a source -- it names 8 bytes, four consecutive columns of one key
  // row -- and a receiver.  Inside a group of 16 lanes, source 4 i + a names key i of four consecutive
  // keys and column block a, and lane 4 a + c receives column 4 a + c of those four keys: the 16 lanes
  // cover 16 consecutive columns (rows of values^T) with four keys each, which is half of the
  // operand.  The key of slot e of contraction step c for lane half hf is 16 c + 8 (e / 4) + 4 hf + e % 4,
  // the order in which the first product leaves P^T in the accumulators.
  const int src16 = lane & 15, src_key = src16 >> 2;
  const int vtr_base = (4 * hf + src_key) * RB + ((2 * ((lane >> 4) & 1) + ((src16 & 3) >> 1)) << 4) + 8 * (src16 & 1);

  // S^T of the wave's queries against key tile t, raw (unscaled) products
  auto scores = [&](auto slot_c, f32x16_t& s) {
    const char* Kt = lds + decltype(slot_c)::value * STAGE;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.0f;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const uint4 a = *reinterpret_cast<const uint4*>(Kt + k_off + (((2 * c + hf) ^ k_x) << 4));
      mma32<T>(s, a, qa[c]);
    }
  };

  // One key tile t, whose raw scores s arrive from the previous step: the mask, the softmax terms,
  // the product with the values -- and the raw scores of tile t + 1, whose matrix instructions stand in
  // the same basic block as the exponentials so that the two run side by side.
  // The exponent's baseline m_run of a query follows the running maximum lazily: it moves only when the
  // maximum has grown by more than ATT_LAZY (in log2 units), so that the accumulated columns are rescaled
  // a few times per query instead of at most tiles; terms are then at most 2^ATT_LAZY, and the quotient
  // O / l does not depend on the baseline.
  auto step = [&](auto slot_c, int t, f32x16_t& s, f32x16_t& s_next) {
    constexpr int SLOT = decltype(slot_c)::value;         // t % NS, known at compile time: the LDS reads of the
    const int j0 = t * 32;                                // tile then take their slot as an immediate offset
    // the mask, by the kind of tile (a wave-uniform choice; only the few lines that apply it differ)
    const int mode = (j0 + 31 <= i0) ? ATT_PLAIN
                     : (j0 > i0 + 31 && bidir && i0 >= img_lo && i0 + 31 < img_hi) ? ATT_AHEAD : ATT_GENERAL;
    if (mode != ATT_PLAIN) {                   // ATT_PLAIN: raw, the scale goes into the exponent below
      // discounts of this lane's 16 keys, staged with the tile
      const char* Bt = lds + SLOT * STAGE + KTILE + VTILE;
      float kbias[16];
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        const float4 x = *reinterpret_cast<const float4*>(Bt + (8 * gq + 4 * hf) * 4);
        kbias[4 * gq] = x.x; kbias[4 * gq + 1] = x.y; kbias[4 * gq + 2] = x.z; kbias[4 * gq + 3] = x.w;
      }
      if (mode == ATT_AHEAD) {
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = fmaf(kbias[v], inv_c2, s[v]);
      } else {
        const bool q_img = bidir && qi >= img_lo && qi < img_hi;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int j = j0 + att_key_of(v, hf);
          const float ahead = q_img ? kbias[v] : -INFINITY;      // a key after the query
          s[v] += (j <= qi ? 0.0f : ahead) * inv_c2;
        }
      }
    }
    float mx = s[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s[v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));        // both lane halves of a query see the same maximum
    // maxima are kept in units of the raw products (finite from the first tile on: key 0 precedes
    // every query)
    const bool moved = mx > m_run + lazy_raw;
    if (__any(moved)) {
      const float m_new = moved ? mx : m_run;
      const float alpha = fast_exp2_att((m_run - m_new) * c2);
      m_run = m_new;
      l_run *= alpha;
      // in place, as assembly: a plain product is hoisted above the branch and the untouched
      // accumulators are then copied register by register on the path that skips it
#pragma unroll
      for (int tt = 0; tt < DT; ++tt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float x = o[tt][v];
          asm volatile("v_mul_f32 %0, %0, %1" : "+v"(x) : "v"(alpha));
          o[tt][v] = x;
        }
    }
    const float m_c = m_run * c2;
    scores(std::integral_constant<int, (SLOT + 1) % NS>{}, s_next);
    float p[16], psum = 0.0f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      p[v] = fast_exp2_att(fmaf(s[v], c2, -m_c));
      psum += p[v];
    }
    l_run += psum;
    uint4 pb[NPS];
#pragma unroll
    for (int c = 0; c < NPS; ++c) pb[c] = att_pack16<T>(&p[c * E]);
    // O^T += V^T_tile P^T: piece 2c + hf of a values^T row holds the keys this lane half has in P^T
    const char* Vt = lds + SLOT * STAGE + KTILE;
#pragma unroll
    for (int c = 0; c < NPS; ++c)
#pragma unroll
      for (int tt = 0; tt < DT; ++tt) {
        uint4 va;
        if constexpr (TR) {
          // row tile tt of values^T = columns 32 tt .. 32 tt + 31 = 16-byte pieces 4 tt .. 4 tt + 3 of a key
          // row, stored in slots (4 tt + x) ^ 4 (key & 3)
          const char* src = Vt + vtr_base + 16 * c * RB + ((tt ^ src_key) << 6);
          const uint2 lo = att_tr_read(src), hi = att_tr_read(src + 8 * RB);
          va = make_uint4(lo.x, lo.y, hi.x, hi.y);
        } else {
          va = *reinterpret_cast<const uint4*>(Vt + v_off[c] + tt * 32 * VB);
        }
        mma32<T>(o[tt], va, pb[c]);
      }
  };

  // Tiles 0 .. PD are requested up front; iteration t requests tile t + 1 + PD and, before its barrier,
  // waits for everything but the newest PD - 1 tiles: tile t + 2 has then landed.  The queries are
  // touched here so that the compiler's wait for their loads stands in front of the loop, not inside
  // it, where it would also wait for the tile requests.
#pragma unroll
  for (int c = 0; c < CH; ++c) asm volatile("" ::"v"(qa[c].x), "v"(qa[c].y), "v"(qa[c].z), "v"(qa[c].w));
  static_assert(NS % 2 == 0, "the two score buffers swap roles every tile, the ring turns every NS tiles");
  static_for<PD + 1>([&](auto t_c) { issue_tile(t_c, decltype(t_c)::value); });
  att_wait_tiles((PD - 1) * my_loads);
  barrier_keep_loads();
  // The loop runs over whole turns of the ring, so that a tile's slot is a compile-time constant, and
  // the raw scores alternate between two register sets instead of being copied.
  f32x16_t s_even, s_odd;
  if (my_tiles > 0) scores(std::integral_constant<int, 0>{}, s_even);
  for (int t0 = 0; t0 < ntiles; t0 += NS) {
    static_for<NS>([&](auto u_c) {
      constexpr int U = decltype(u_c)::value;
      const int t = t0 + U;
      if (t < ntiles) {                        // the same for every wave of the workgroup
        issue_tile(std::integral_constant<int, (U + 1 + PD) % NS>{}, t + 1 + PD);
        if (t < my_tiles) {
          if constexpr (U % 2 == 0) step(u_c, t, s_even, s_odd);
          else step(u_c, t, s_odd, s_even);
        }
        att_wait_tiles((PD - 1) * my_loads);
        barrier_keep_loads();
      }
    });
  }
  wait_all_vmem();                             // the surplus requests of the last iterations

  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = 1.0f / l_tot;
  if (qi < N) {
    T* orow = out + (((int64_t)b * H + h) * N + qi) * D;
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

// bf16 values with d = 128 are read as they are; every other case goes through a transposed copy
static bool att_row_major_values(const asap_params& p) { return p.qk_dtype == ASAP_BF16 && p.d == 128; }

size_t attention_workspace_bytes(const asap_params& p) {
  const size_t es = p.qk_dtype == ASAP_BF16 ? 2 : 4;
  const size_t vt = att_row_major_values(p) ? 0 : align256(es * (size_t)p.B * p.Hkv * p.d * att_npad(p));
  return vt + align256(sizeof(float) * (size_t)p.B * att_npad(p));
}

template <typename T>
static hipError_t attention_typed(const asap_params& p, const void* q, Strides3 sq, const void* k, Strides3 sk,
                                  const void* v, Strides3 sv, const float* s_hat, void* out, char* ws,
                                  hipStream_t st, Timer* tm) {
  constexpr int E = elem<T>::per16;
  const int N = p.P + p.V + p.Tmax, Npad = att_npad(p);
  const bool row_major_values = att_row_major_values(p);    // the kernel transposes while it reads LDS
  T* vt = reinterpret_cast<T*>(ws);                         // (not used then)
  float* bias2 = reinterpret_cast<float*>(
      ws + (row_major_values ? 0 : align256(sizeof(T) * (size_t)p.B * p.Hkv * p.d * Npad)));
  const bool bidir = p.mask_mode == ASAP_MASK_KEYBIAS;
  // (with the mask off the table is -inf everywhere and s_hat is not read)
  ASAP_LAUNCH(tm, "k_att_bias", k_att_bias, dim3((Npad + 255) / 256, p.B), dim3(256), 0, st, bidir ? s_hat : nullptr,
              p.P, p.V, Npad, p.lambda_max, p.eps, bias2);
  if (!row_major_values)
    ASAP_LAUNCH(tm, "k_vtranspose", k_vtranspose<T>, dim3(Npad / 32, p.Hkv, p.B), dim3(256), 0, st,
                static_cast<const T*>(v), sv, N, Npad, p.d, vt);
  const float c2 = 1.4426950408889634f / sqrtf((float)p.d);
  const dim3 grid((N + ATT_QWG - 1) / ATT_QWG, p.H, p.B);
  const int ch = p.d / E / 2;
  constexpr int PD = ATT_PD;                   // key tiles requested ahead
  const size_t lds = (PD + 2) * ((size_t)(32 * 32 * ch + p.d * 32 * sizeof(T)) + ATT_BIASB);
#define ASAP_ATT(CHV)                                                                                          \
  do {                                                                                                         \
    auto kern = k_attention<T, CHV, PD>;                                                                                    \
    if (lds > 48 * 1024) {                                                                                     \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                  \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                \
      if (e != hipSuccess) return e;                                                                           \
    }                                                                                                          \
    ASAP_LAUNCH(tm, "k_attention", kern, grid, dim3(64 * ATT_NW), lds, st, static_cast<const T*>(q), sq,       \
                static_cast<const T*>(k), sk, vt, Npad, static_cast<const T*>(v), sv, bias2, bidir ? 1 : 0,    \
                static_cast<T*>(out), p.H,                                                                      \
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
