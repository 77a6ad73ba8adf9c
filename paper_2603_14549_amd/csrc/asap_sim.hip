// Cosine routing of pruned tokens to kept tokens (Sec. 4.2): the one dense contraction of the
// stage, (pruned rows) x (kept rows)^T over the hidden dimension, on the matrix cores, with the
// row arg-max fused into the epilogue.
//
//   k_sim<T, NT>  (bf16 hidden states)
//                 workgroup tile BM = 128 source rows x BN = 64*NT destination rows, 256 threads =
//                 4 waves (2 x 2 over the tile, each 64 x 32*NT = 2 x NT MFMA tiles of 32 x 32), one
//                 wave per SIMD so that a wave may use the whole 512-entry register file.  The
//                 hidden dimension is walked in steps of 128 bytes per row, one barrier per step.
//                 Operands reach LDS by direct global -> LDS loads (no registers in between) that
//                 every wave issues between its MFMAs; the squared norms of the rows are added up
//                 from the operands a wave holds, also in the shadow of the MFMAs (waves that hold
//                 the same rows take half of the contraction slices each).
//                 The source rows are read once, from HBM, so their 128 x 128 B slices go through a
//                 ring of 4 LDS slots and are asked for three steps ahead; the destination rows are
//                 shared by all tiles of an image and come from L2, so two slots (one step ahead)
//                 are enough for their BN x 128 B slices at the widest tile; narrower tiles leave
//                 room for deeper rings (sim_na, sim_nb).
//                 LDS rows are unpadded; the 16-byte piece p of row r is stored in slot
//                 p ^ ((r >> 1) & 7): any 16 consecutive rows then cover all 64 banks once, for the
//                 1 KiB-contiguous loads as well as for the strided 16-byte operand reads.
//                 The grid is one-dimensional and XCD-aware: consecutive workgroup ids go to the 8
//                 XCDs round-robin, so id % 8 picks the XCD and all tiles of one image are given
//                 ids with the same id % 8 -- they then share that XCD's L2 for the kept panel
//                 (batches of fewer than 8 images spread an image over several XCDs instead).
//                 A workgroup takes one destination tile.  When the destination rows need several
//                 (k > 64*NT), the tiles of a source tile are workgroups of their own: each leaves
//                 its row winner as a 64-bit key (order-preserving value bits, then the inverted
//                 column so that equal values keep the smaller column) in a slot of its own.
//                 Launches of at most 128 workgroups also cut the hidden dimension into slices
//                 with workgroups of their own, which leave raw partial products and partial
//                 squared norms instead of a row winner.
//   k_sim_f32<NT> (f32 hidden states) the same tile, grid and epilogue; every value is cut into three
//                 bf16 pieces once per workgroup on its way global memory -> registers -> LDS, and the
//                 waves multiply finished pieces (six piece products per pair of values)
//   k_sim_finish  largest key of a row -> assign, best_sim (threshold and source norm applied here)
//   k_sim_reduce  sums the slices of a split launch, then the same scaling, predicate and arg-max
#include "asap_device.hpp"
#include "asap_launch.hpp"
#include "asap_select.hpp"

namespace asap {

constexpr int SIM_BM = 128;
constexpr int SIM_ROWB = 128;      // bytes of a row held in LDS per step
constexpr int NUM_XCD = 8;
// LDS ring slots for the source rows (NA) and the destination rows (NB) by tile width: as deep as
// 160 KiB allow, NA > NB >= 2.  Narrow tiles belong to launches with few workgroups (small batches, the
// search inside the kept set), whose steps last as long as a load takes to arrive divided by how many
// steps ahead it was asked for.
constexpr int sim_na(int nt) { return nt == 1 ? 6 : nt == 2 ? 5 : 4; }
constexpr int sim_nb(int nt) { return nt == 1 ? 4 : nt <= 3 ? 3 : 2; }

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// Sum of squares of the elements of a 16-byte chunk, kept in four independent partial sums so that
// consecutive operations never wait for each other.
struct SumSq4 {
  float p[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  __device__ __forceinline__ float total() const { return (p[0] + p[1]) + (p[2] + p[3]); }
};
template <typename T> __device__ __forceinline__ void sumsq16(const uint4& c, SumSq4& acc);
template <> __device__ __forceinline__ void sumsq16<bf16_t>(const uint4& c, SumSq4& acc) {
  bf16x2_t p;
  __builtin_memcpy(&p, &c.x, 4); acc.p[0] = __builtin_amdgcn_fdot2_f32_bf16(p, p, acc.p[0], false);
  __builtin_memcpy(&p, &c.y, 4); acc.p[1] = __builtin_amdgcn_fdot2_f32_bf16(p, p, acc.p[1], false);
  __builtin_memcpy(&p, &c.z, 4); acc.p[2] = __builtin_amdgcn_fdot2_f32_bf16(p, p, acc.p[2], false);
  __builtin_memcpy(&p, &c.w, 4); acc.p[3] = __builtin_amdgcn_fdot2_f32_bf16(p, p, acc.p[3], false);
}
template <> __device__ __forceinline__ void sumsq16<float>(const uint4& c, SumSq4& acc) {
  float f[4];
  unpack16<float>(c, f);
  acc.p[0] = fmaf(f[0], f[0], acc.p[0]); acc.p[1] = fmaf(f[1], f[1], acc.p[1]);
  acc.p[2] = fmaf(f[2], f[2], acc.p[2]); acc.p[3] = fmaf(f[3], f[3], acc.p[3]);
}

// all-reduce over a row of 16 lanes by rotations inside the row (the caller joins the two rows of a
// 32-lane half with one exchange)
template <int CTRL> __device__ __forceinline__ uint32_t dpp_u32(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, CTRL, 0xF, 0xF, false);
}
__device__ __forceinline__ float rowmax16(float x) {
  x = fmaxf(x, __uint_as_float(dpp_u32<0x128>(__float_as_uint(x))));   // row_ror:8
  x = fmaxf(x, __uint_as_float(dpp_u32<0x124>(__float_as_uint(x))));   // row_ror:4
  x = fmaxf(x, __uint_as_float(dpp_u32<0x122>(__float_as_uint(x))));   // row_ror:2
  x = fmaxf(x, __uint_as_float(dpp_u32<0x121>(__float_as_uint(x))));   // row_ror:1
  return x;
}
__device__ __forceinline__ int rowmin16(int x) {
  x = min(x, (int)dpp_u32<0x128>((uint32_t)x));
  x = min(x, (int)dpp_u32<0x124>((uint32_t)x));
  x = min(x, (int)dpp_u32<0x122>((uint32_t)x));
  x = min(x, (int)dpp_u32<0x121>((uint32_t)x));
  return x;
}

// What a workgroup knows about its tile once the products are done, and where the results go.
struct SimTile {
  int b, B, M, k, V;
  int m0, n0;                 // first source row, first destination column
  int pass, ptiles, mt;       // destination tile, their count, source tile
  int ks, ksplit;             // slice of the hidden dimension
  float threshold;
  const int32_t* kept;
  const float* s_hat;
  int32_t* assign;
  float* best_sim;
  unsigned long long* best_key;
  float* src_norm2;
  float* dots;
  float* kept_norm2;
};

// Epilogue of a 128 x 64 NT tile held as 2 x NT accumulators per wave (waves 2 x 2 over the tile):
// norm2 [128] / normk [64 NT] hold the squared norms of its rows / columns (this slice's share),
// part [2][128] is LDS scratch, srow [128] the salience of the source rows (ANCHORED).  The caller
// has put a barrier after the writes of norm2, normk and srow.
template <int NT, bool ANCHORED>
__device__ __forceinline__ void sim_tile_epilogue(f32x16_t (&acc)[2][NT], const float* norm2, const float* normk,
                                                  uint2* part, const float* srow, const SimTile& T_) {
  constexpr int BN = 64 * NT;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31;
  const int wm = wave >> 1, wn = wave & 1;
  const int b = T_.b, B = T_.B, M = T_.M, k = T_.k, V = T_.V, m0 = T_.m0, n0 = T_.n0, pass = T_.pass;
  const int ptiles = T_.ptiles, mt = T_.mt, ks = T_.ks, ksplit = T_.ksplit;
  const float threshold = T_.threshold;
  const int32_t* __restrict__ kept = T_.kept;
  const float* __restrict__ s_hat = T_.s_hat;
  float run_v = -INFINITY;   // best of this workgroup's destination tile (threads < BM)
  int run_c = 0;
  {
    if (ksplit > 1) {
      // this slice's share of the products and of the squared norms; k_sim_reduce adds the slices up
      const int64_t img = (int64_t)ks * B + b;
      if (pass == 0 && tid < SIM_BM && m0 + tid < M) T_.src_norm2[img * M + m0 + tid] = norm2[tid];
      if (mt == 0)
        for (int c = tid; c < BN; c += 256)        // BN may exceed the workgroup size
          if (n0 + c < k) T_.kept_norm2[img * k + n0 + c] = normk[c];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = m0 + wm * 64 + i * 32 + mma32_row(v, lane);
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            const int col = n0 + wn * (BN / 2) + t * 32 + n;
            if (row < M && col < k) T_.dots[(img * M + row) * k + col] = acc[i][t][v];
          }
        }
      return;
    }

    // Row arg-max of dot / |x_j| over this pass's destinations (|x_i| > 0 does not move it).
    // A lane first takes the best of its NT columns of a row (columns past k get -inf), then the 32
    // lanes that share the row agree on the maximum and on the smallest column that reaches it.
    float invk[NT], bias[NT];
    int colv[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int cl = wn * (BN / 2) + t * 32 + n;
      colv[t] = n0 + cl;
      const bool valid = colv[t] < k;
      invk[t] = valid ? 1.0f / fmaxf(sqrtf(normk[cl]), 1e-8f) : 0.0f;
      bias[t] = valid ? 0.0f : -INFINITY;
    }
    float scol[NT];            // ANCHORED: salience of this lane's destination columns
#pragma unroll
    for (int t = 0; t < NT; ++t)
      scol[t] = (ANCHORED && colv[t] < k) ? s_hat[(int64_t)b * V + kept[(int64_t)b * k + colv[t]]] : 0.0f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      // stage by stage over the 16 rows a lane holds, so that the cross-lane exchanges of
      // different rows overlap instead of waiting for one another
      float bv[16], mv[16], ov[16];
      int bc[16], mc[16], oc[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float c[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) c[t] = fmaf(acc[i][t][v], invk[t], bias[t]);
        if (ANCHORED) {
          const int rloc = wm * 64 + i * 32 + mma32_row(v, lane);
          const float sr_ = srow[rloc];
          const int rslot = m0 + rloc;
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            const bool stronger = (scol[t] > sr_) | ((scol[t] == sr_) & (colv[t] < rslot));
            c[t] = stronger ? c[t] : -INFINITY;
          }
        }
        bv[v] = c[0];
#pragma unroll
        for (int t = 1; t < NT; ++t) bv[v] = fmaxf(bv[v], c[t]);
        bc[v] = 0x7fffffff;
#pragma unroll
        for (int t = NT - 1; t >= 0; --t) bc[v] = (c[t] == bv[v]) ? colv[t] : bc[v];   // columns ascend with t
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) mv[v] = rowmax16(bv[v]);
#pragma unroll
      for (int v = 0; v < 16; ++v) ov[v] = __shfl_xor(mv[v], 16);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        mv[v] = fmaxf(mv[v], ov[v]);
        mc[v] = rowmin16(bv[v] == mv[v] ? bc[v] : 0x7fffffff);
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) oc[v] = __shfl_xor(mc[v], 16);
      if (n == 0) {
#pragma unroll
        for (int v = 0; v < 16; ++v)
          part[wn * SIM_BM + wm * 64 + i * 32 + mma32_row(v, lane)] =
              make_uint2(__float_as_uint(mv[v]), (uint32_t)min(mc[v], oc[v]));
      }
    }
    __syncthreads();
    if (tid < SIM_BM) {
      uint2 p0 = part[tid], p1 = part[SIM_BM + tid];
      float v0 = __uint_as_float(p0.x), v1 = __uint_as_float(p1.x);
      int c0 = (int)p0.y, c1 = (int)p1.y;
      if (v1 > v0 || (v1 == v0 && c1 < c0)) { v0 = v1; c0 = c1; }
      run_v = v0;
      run_c = c0;
    }
  }
  if (tid < SIM_BM && m0 + tid < M) {
    const int64_t o = (int64_t)b * M + m0 + tid;
    if (ptiles == 1) {
      float c = run_v / fmaxf(sqrtf(norm2[tid]), 1e-8f);
      T_.best_sim[o] = c;
      T_.assign[o] = (c > threshold) ? run_c : -1;
    } else {
      // several destination tiles per source row: every tile leaves its best as a 64-bit key (value,
      // then the inverted column so that equal values keep the smaller column); k_sim_finish takes the
      // largest key of a row and turns it into assign / best_sim
      const unsigned long long key = ((unsigned long long)float_key(run_v) << 32) | (0xFFFFFFFFu - (uint32_t)run_c);
      T_.best_key[(int64_t)pass * ((int64_t)B * M) + o] = key;
      if (pass == 0) T_.src_norm2[o] = norm2[tid];
    }
  }
}

// ANCHORED (the routing inside the kept set, Sec. 4.2): the source rows are the kept tokens too
// (pruned == kept, M == k), and a destination counts for a source only if it is the stronger of the
// two: larger salience s_hat, ties to the smaller index -- which is the smaller slot, both lists
// being ascending.  A token is never its own destination.
template <typename T, int NT, bool ANCHORED>
__global__ __launch_bounds__(256) void k_sim(const T* __restrict__ xv, int64_t sb, int64_t sr, int D,
                                              const int32_t* __restrict__ pruned, const int32_t* __restrict__ kept,
                                              const float* __restrict__ s_hat, int V, int B, int M, int k,
                                              int mtiles, int ptiles, int spread, int vmt, float threshold,
                                              int32_t* __restrict__ assign,
                                              float* __restrict__ best_sim, unsigned long long* __restrict__ best_key,
                                              float* __restrict__ src_norm2, int ksplit, float* __restrict__ dots,
                                              float* __restrict__ kept_norm2) {
  constexpr int BN = 64 * NT;
  constexpr int PA = SIM_BM / 32;                // source-row loads a thread issues per step
  constexpr int PB = BN / 32;                    // destination-row loads
  constexpr int ASTAGE = SIM_BM * SIM_ROWB, BSTAGE = BN * SIM_ROWB;
  constexpr int NA = sim_na(NT), NB = sim_nb(NT);
  static_assert(NA > NB && NB >= 2, "ring depths");
  static_assert(PA + PB <= 8 * NT, "one load per MFMA slot");
  extern __shared__ __align__(16) char lds[];
  char* ldsB = lds + NA * ASTAGE;
  const uint32_t lds_addr = lds_address(lds), ldsB_addr = lds_addr + NA * ASTAGE;
  float* norm2 = reinterpret_cast<float*>(ldsB + NB * BSTAGE);   // [BM] squared norms of the source rows
  float* normk = norm2 + SIM_BM;                                 // [BN] squared norms of this pass's kept rows
  uint2* part = reinterpret_cast<uint2*>(normk + BN);            // [2][BM] (value, column) per column half
  float* srow = reinterpret_cast<float*>(part + 2 * SIM_BM);     // [BM] salience of the source rows (ANCHORED)

  // XCD-aware decode of the linear workgroup id
  // (a workgroup = one source tile x one destination tile; the destination tiles of a source tile
  // are neighbours in the id order)
  // With fewer than 8 images one image per XCD would leave XCDs idle: an image's source tiles are then
  // dealt to `spread` XCDs (tile mt to the XCD of "virtual image" b * spread + mt % spread), each of
  // which keeps its own copy of the image's destination panel in L2.
  // With ksplit > 1 (launches that would leave most of the chip idle) the hidden dimension is cut into
  // ksplit slices, each with workgroups of its own, which leave raw partial products and partial
  // squared norms for k_sim_reduce instead of taking the arg-max themselves.
  const int xcd = blockIdx.x % NUM_XCD, slot_p = blockIdx.x / NUM_XCD;
  const int pass = slot_p % ptiles, ks = (slot_p / ptiles) % ksplit, slot = slot_p / (ptiles * ksplit);
  const int vb = (slot / vmt) * NUM_XCD + xcd;
  const int b = vb / spread;
  const int mt = vb % spread + spread * (slot % vmt);
  if (b >= B || mt >= mtiles) return;
  const int m0 = mt * SIM_BM;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, hf = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  const char* xb = reinterpret_cast<const char*>(xv + b * sb);
  const int64_t rowb = sr * (int64_t)sizeof(T);
  const int steps = (D * (int)sizeof(T)) / SIM_ROWB / ksplit;     // ksplit divides the step count
  const int step_lo = ks * steps;
  // Every workgroup walks its part of the hidden dimension from its own starting step: rows are a
  // power-of-two number of bytes apart, so workgroups in lockstep would all hit the same memory channel.
  const int rot = (mt + 16 * (slot / vmt)) % steps;
  auto step_base = [&](int s) {
    int sr_ = s + rot;
    if (sr_ >= steps) sr_ -= steps;
    return xb + (int64_t)(step_lo + sr_) * SIM_ROWB;
  };

  // Loads: thread (rr, q) fetches, for rows rr + 32 i, the piece that belongs in slot q of the row;
  // one load instruction of wave w fills rows 8 w .. 8 w + 7 of a 32-row block, 1 KiB contiguous.
  const int rr = tid >> 3, q = tid & 7;
  const uint32_t piece_off = (uint32_t)((q ^ ((rr >> 1) & 7)) * 16);
  uint32_t offa[PA], offb[PB];      // byte offsets from the image base (an image spans < 4 GiB)
#pragma unroll
  for (int i = 0; i < PA; ++i) {
    int r = min(m0 + rr + 32 * i, M - 1);
    offa[i] = (uint32_t)(pruned[(int64_t)b * M + r] * rowb) + piece_off;
  }
  // Operand reads: byte offset, inside its row, of the chunk this lane reads at position kk of a step.
  // Wave w walks the four contraction slices of a step in the order kk ^ w.  The products do not care,
  // and the sums for the norms can then be shared without a branch: every wave adds up the destination
  // chunks at positions 0 and 1 and the source chunks at positions 0 and 2; the wave below (w ^ 2, same
  // destination rows) covers the other two slices of the former, the wave beside (w ^ 1, same source
  // rows) those of the latter, and the halves meet in LDS after the last step.
  int sw[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) sw[kk] = ((hf * 4 + (kk ^ wave)) ^ ((n >> 1) & 7)) * 16;

  if (ANCHORED) {            // the barriers of the fill below make these visible
    if (tid < SIM_BM) srow[tid] = s_hat[(int64_t)b * V + pruned[(int64_t)b * M + min(m0 + tid, M - 1)]];
  }
  {
    const int n0 = pass * BN;
#pragma unroll
    for (int j = 0; j < PB; ++j) {
      int c = min(n0 + rr + 32 * j, k - 1);
      offb[j] = (uint32_t)(kept[(int64_t)b * k + c] * rowb) + piece_off;
    }
    f32x16_t acc[2][NT];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][t][v] = 0.0f;
    SumSq4 ss_a[2], ss_b[NT];

    // fill: destination slices 0 .. NB-2, source slices 0 .. NA-2
    {
#pragma unroll
      for (int a = 0; a < NB - 1; ++a) {
        if (a < steps) {
          const char* g = step_base(a);
#pragma unroll
          for (int j = 0; j < PB; ++j)
            load_to_lds16(g, offb[j], ldsB_addr + a * BSTAGE + (8 * wave + 32 * j) * SIM_ROWB);
        }
      }
#pragma unroll
      for (int a = 0; a < NA - 1; ++a) {
        if (a < steps) {
          const char* ga = step_base(a);
#pragma unroll
          for (int i = 0; i < PA; ++i)
            load_to_lds16(ga, offa[i], lds_addr + a * ASTAGE + (8 * wave + 32 * i) * SIM_ROWB);
        }
      }
      wait_all_vmem();
      __syncthreads();
    }

    int sa = 0, sb_ = 0;       // ring slots of the current step: s % NA, s % NB
    for (int s = 0; s < steps; ++s) {
      // During step s the waves read source slot s % NA and destination slot s % NB.  Meanwhile the
      // destination rows of step s+NB-1 are asked for first, then the source rows of step s+NA-1, each
      // into the slot the previous step has just left.  Loads retire in order, so what step s+1 needs
      // has landed once nothing older than the source loads of step s-NB+2 is outstanding: those PA
      // loads and the PA+PB loads of each of the NB-2 steps since.
      const char* A = lds + sa * ASTAGE + (wm * 64 + n) * SIM_ROWB;
      const char* Bp = ldsB + sb_ * BSTAGE + (wn * (BN / 2) + n) * SIM_ROWB;
      // Past the last step the loads repeat the current step into a slot nobody reads any more:
      // cheaper than branches around every load, which would also split the schedule below.
      const char* gb = step_base(s + NB - 1 < steps ? s + NB - 1 : s);
      const char* ga = step_base(s + NA - 1 < steps ? s + NA - 1 : s);
      const uint32_t db = ldsB_addr + (sb_ == 0 ? NB - 1 : sb_ - 1) * BSTAGE + (8 * wave) * SIM_ROWB;
      const uint32_t da = lds_addr + (sa == 0 ? NA - 1 : sa - 1) * ASTAGE + (8 * wave) * SIM_ROWB;
      sa = sa + 1 == NA ? 0 : sa + 1;
      sb_ = sb_ + 1 == NB ? 0 : sb_ + 1;
      auto load_unit = [&](int u) {      // the u-th load of this step, if there is one
        if (u < PB) load_to_lds16(gb, offb[u < PB ? u : 0], db + u * 32 * SIM_ROWB);
        else if (u < PB + PA) load_to_lds16(ga, offa[u < PB + PA ? u - PB : 0], da + (u - PB) * 32 * SIM_ROWB);
      };
      // LDS operand reads run one contraction slice ahead of the MFMAs that use them
      uint4 a[2][2], bq[2][NT];
      auto load_op = [&](int set, int kk, int u) {      // in the order the MFMAs need them
        if (u == 0) a[set][0] = *reinterpret_cast<const uint4*>(A + sw[kk]);
        else if (u == 2) a[set][1] = *reinterpret_cast<const uint4*>(A + 32 * SIM_ROWB + sw[kk]);
        else {
          const int t = u == 1 ? 0 : u - 2;
          if (t < NT) bq[set][t] = *reinterpret_cast<const uint4*>(Bp + t * 32 * SIM_ROWB + sw[kk]);
        }
      };
#pragma unroll
      for (int u = 0; u < NT + 2; ++u) load_op(0, 0, u);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        // After each MFMA: one LDS read for the next contraction slice, one global -> LDS load and a
        // few dot products for the norms, all in the MFMA's shadow.
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          __builtin_amdgcn_sched_barrier(0);
          mma32<T>(acc[0][t], a[kk & 1][0], bq[kk & 1][t]);
          if (kk < 3) load_op((kk + 1) & 1, kk + 1, 2 * t);
          if (kk < 2) sumsq16<T>(bq[kk & 1][t], ss_b[t]);
          load_unit(kk * 2 * NT + 2 * t);
          __builtin_amdgcn_sched_barrier(0);
          mma32<T>(acc[1][t], a[kk & 1][1], bq[kk & 1][t]);
          if (kk < 3) load_op((kk + 1) & 1, kk + 1, 2 * t + 1);
          if ((kk & 1) == 0) {
            if (t == 0) sumsq16<T>(a[kk & 1][0], ss_a[0]);
            if (t == 1 || NT == 1) sumsq16<T>(a[kk & 1][1], ss_a[1]);
          }
          load_unit(kk * 2 * NT + 2 * t + 1);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (kk < 3) {
#pragma unroll
          for (int u = 2 * NT; u < NT + 2; ++u) load_op((kk + 1) & 1, kk + 1, u);     // NT == 1 only
        }
      }
      wait_vmem_but<PA + (NB - 2) * (PA + PB)>();
      barrier_keep_loads();
    }

    wait_all_vmem();   // the repeated loads of the last steps
    // The two lane halves hold the two halves of every 128-byte slice, and the wave beside (source
    // rows) or below (destination rows) the other two contraction slices of every step: it adds its
    // half in a second turn.
#pragma unroll
    for (int turn = 0; turn < 2; ++turn) {
      if (wn == turn) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          float v = ss_a[i].total();
          v += __shfl_xor(v, 32);
          float* o = &norm2[wm * 64 + i * 32 + n];
          if (hf == 0) *o = turn == 0 ? v : *o + v;
        }
      }
      if (wm == turn) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          float v = ss_b[t].total();
          v += __shfl_xor(v, 32);
          float* o = &normk[wn * (BN / 2) + t * 32 + n];
          if (hf == 0) *o = turn == 0 ? v : *o + v;
        }
      }
      __syncthreads();   // after the second turn: norms visible
    }

    SimTile tile;
    tile.b = b; tile.B = B; tile.M = M; tile.k = k; tile.V = V; tile.m0 = m0; tile.n0 = n0; tile.pass = pass;
    tile.ptiles = ptiles; tile.mt = mt; tile.ks = ks; tile.ksplit = ksplit; tile.threshold = threshold;
    tile.kept = kept; tile.s_hat = s_hat; tile.assign = assign; tile.best_sim = best_sim; tile.best_key = best_key;
    tile.src_norm2 = src_norm2; tile.dots = dots; tile.kept_norm2 = kept_norm2;
    sim_tile_epilogue<NT, ANCHORED>(acc, norm2, normk, part, srow, tile);
  }
}

// f32 hidden states.  The bf16 matrix instructions take three bf16 pieces per value (hi + mid + lo =
// the value to 2^-27) and a product is the sum of the six piece products that matter -- a third of
// the matrix time of the f32 instruction.  Cutting a value into its pieces costs about five vector
// instructions, and a wave that issues those for every operand it multiplies (its 64 source and 32 NT
// destination rows, which the wave beside or below cuts again) is bound by its own instruction stream,
// not by the matrix cores.  So here every value is cut exactly once per workgroup: the rows travel
// global memory -> registers (asked for two steps ahead) -> pieces -> LDS, each thread cutting 8
// consecutive values of 2 + NT rows per step, and the waves read finished pieces as operands.  LDS
// holds the pieces of two steps (one being multiplied, one being written); one barrier per step.
//   LDS row of a step: 208 bytes = hi | mid | lo planes of 64 bytes (32 values x 2 bytes) + 16 bytes
//   of padding: 16 consecutive rows then start in 16 different groups of 4 banks.
// Tile, waves, grid order, slices of the hidden dimension and epilogue are those of k_sim.
constexpr int SIMF_ROWP = 208;
constexpr int SIMF_MAX_NT = 4;      // 2 x (128 + 256) rows x 208 bytes = 156 KiB
template <int NT, bool ANCHORED>
__global__ __launch_bounds__(256) void k_sim_f32(const float* __restrict__ xv, int64_t sb, int64_t sr, int D,
                                                  const int32_t* __restrict__ pruned,
                                                  const int32_t* __restrict__ kept, const float* __restrict__ s_hat,
                                                  int V, int B, int M, int k, int mtiles, int ptiles, int spread,
                                                  int vmt, float threshold, int32_t* __restrict__ assign,
                                                  float* __restrict__ best_sim,
                                                  unsigned long long* __restrict__ best_key,
                                                  float* __restrict__ src_norm2, int ksplit,
                                                  float* __restrict__ dots, float* __restrict__ kept_norm2) {
  constexpr int BN = 64 * NT;
  constexpr int ROWS = SIM_BM + BN;              // rows of a step in LDS: sources, then destinations
  constexpr int NJ = ROWS / 64;                  // rows a thread cuts per step (8 values of each)
  constexpr int STAGE = ROWS * SIMF_ROWP;
  extern __shared__ __align__(16) char lds[];
  // the epilogue's arrays take the place of the pieces once the last step is through
  float* norm2 = reinterpret_cast<float*>(lds);                  // [BM]
  float* normk = norm2 + SIM_BM;                                 // [BN]
  uint2* part = reinterpret_cast<uint2*>(normk + BN);            // [2][BM]
  float* srow = reinterpret_cast<float*>(part + 2 * SIM_BM);     // [BM]

  const int xcd = blockIdx.x % NUM_XCD, slot_p = blockIdx.x / NUM_XCD;
  const int pass = slot_p % ptiles, ks = (slot_p / ptiles) % ksplit, slot = slot_p / (ptiles * ksplit);
  const int vb = (slot / vmt) * NUM_XCD + xcd;
  const int b = vb / spread;
  const int mt = vb % spread + spread * (slot % vmt);
  if (b >= B || mt >= mtiles) return;
  const int m0 = mt * SIM_BM, n0 = pass * BN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, hf = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  const char* xb = reinterpret_cast<const char*>(xv + b * sb);
  const int64_t rowb = sr * (int64_t)sizeof(float);
  const int steps = (D * (int)sizeof(float)) / SIM_ROWB / ksplit;     // ksplit divides the step count
  const int step_lo = ks * steps;
  const int rot = (mt + 16 * (slot / vmt)) % steps;                   // see k_sim
  auto step_base = [&](int s) __attribute__((always_inline)) {
    int sr_ = s + rot;
    if (sr_ >= steps) sr_ -= steps;
    return xb + (int64_t)(step_lo + sr_) * SIM_ROWB;
  };

  // Cutting: thread (lr, g4) takes the values 8 g4 .. 8 g4 + 7 of the step for rows lr + 64 j.
  const int lr = tid >> 2, g4 = tid & 3;
  uint32_t off[NJ];           // byte offsets from the image base (an image spans < 4 GiB)
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int row = lr + 64 * j;
    const int idx = row < SIM_BM ? pruned[(int64_t)b * M + min(m0 + row, M - 1)]
                                 : kept[(int64_t)b * k + min(n0 + row - SIM_BM, k - 1)];
    off[j] = (uint32_t)(idx * rowb) + g4 * 32;
  }
  const int wr = lr * SIMF_ROWP + g4 * 16;        // where the thread's pieces of row lr go (+ 64 j rows)
  // Operands: lane (n, hf) reads the values 16 kb + 8 hf .. + 7 of its rows for contraction block kb.
  const int rd_a = (wm * 64 + n) * SIMF_ROWP + hf * 16;
  const int rd_b = (SIM_BM + wn * (BN / 2) + n) * SIMF_ROWP + hf * 16;

  f32x16_t acc[2][NT];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][t][v] = 0.0f;
  SumSq4 ss[NJ];              // squared norms of the thread's share of its rows

  uint4 raw[2][NJ][2];        // the values of two steps on their way
  auto fetch = [&](uint4 (&r)[NJ][2], int s) __attribute__((always_inline)) {
    const char* g = step_base(s);
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      r[j][0] = ldg16(g + off[j]);
      r[j][1] = ldg16(g + off[j] + 16);
    }
  };
  auto cut = [&](const uint4 (&r)[NJ][2], char* stage) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const Split3 p3 = split_f32x8(r[j][0], r[j][1]);
      sumsq16<float>(r[j][0], ss[j]);
      sumsq16<float>(r[j][1], ss[j]);
      char* dst = stage + wr + j * 64 * SIMF_ROWP;
      *reinterpret_cast<uint4*>(dst) = p3.hi;
      *reinterpret_cast<uint4*>(dst + 64) = p3.mid;
      *reinterpret_cast<uint4*>(dst + 128) = p3.lo;
    }
  };
  // The same cut in NJ x 11 units, for a schedule written out by hand: per row of the thread, 8 units
  // that take one value pair through one of the two phases of split_pair, 2 units of squared norms,
  // and the unit that stores the three pieces and asks for the row's values two steps on (gnext: where
  // that step starts), so that every load has almost two steps to arrive.  The pieces under way live
  // in p3, r0, r1.
  constexpr int CUT_UNITS = NJ * 11;
  Split3 p3;
  float r0 = 0.0f, r1 = 0.0f;
  auto cut_unit = [&](auto uc, uint4 (&r)[NJ][2], char* stage, const char* gnext) __attribute__((always_inline)) {
    constexpr int U = decltype(uc)::value;
    constexpr int J = U / 11, R = U % 11;
    if constexpr (R < 8) {
      constexpr int Q = R / 2;
      auto put = [](uint4& v, uint32_t x) __attribute__((always_inline)) {
        if constexpr (Q == 0) v.x = x;
        else if constexpr (Q == 1) v.y = x;
        else if constexpr (Q == 2) v.z = x;
        else v.w = x;
      };
      if constexpr (R % 2 == 0) {
        const uint4& c = r[J][Q / 2];
        const float a = __uint_as_float(Q % 2 == 0 ? c.x : c.z), b = __uint_as_float(Q % 2 == 0 ? c.y : c.w);
        const uint32_t hi = pk_bf16(a, b);
        r0 = a - __uint_as_float(hi << 16);
        r1 = b - __uint_as_float(hi & 0xffff0000u);
        put(p3.hi, hi);
      } else {
        const uint32_t mid = pk_bf16(r0, r1);
        put(p3.mid, mid);
        put(p3.lo, pk_bf16(r0 - __uint_as_float(mid << 16), r1 - __uint_as_float(mid & 0xffff0000u)));
      }
    } else if constexpr (R < 10) {
      sumsq16<float>(r[J][R - 8], ss[J]);
    } else {
      char* dst = stage + wr + J * 64 * SIMF_ROWP;
      *reinterpret_cast<uint4*>(dst) = p3.hi;
      *reinterpret_cast<uint4*>(dst + 64) = p3.mid;
      *reinterpret_cast<uint4*>(dst + 128) = p3.lo;
      r[J][0] = ldg16(gnext + off[J]);
      r[J][1] = ldg16(gnext + off[J] + 16);
    }
  };
  // Operand pieces of contraction block kb (16 values) of the stage
  Split3 a3[2], b3[NT];
  auto operands = [&](const char* stage, int kb) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const char* p = stage + rd_a + i * 32 * SIMF_ROWP + kb * 32;
      a3[i].hi = *reinterpret_cast<const uint4*>(p);
      a3[i].mid = *reinterpret_cast<const uint4*>(p + 64);
      a3[i].lo = *reinterpret_cast<const uint4*>(p + 128);
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const char* p = stage + rd_b + t * 32 * SIMF_ROWP + kb * 32;
      b3[t].hi = *reinterpret_cast<const uint4*>(p);
      b3[t].mid = *reinterpret_cast<const uint4*>(p + 64);
      b3[t].lo = *reinterpret_cast<const uint4*>(p + 128);
    }
  };
  // A step, slot by slot and in this order (the compiler moves nothing across a slot's end): one piece
  // product -- product by product over the 2 NT accumulators, so that neighbouring matrix instructions
  // never wait for one another -- and that slot's share of the cut of the next step's values, a few
  // vector instructions that run in the matrix instruction's shadow.  CUT = false: the last step.
  constexpr int SLOTS = 24 * NT;
  auto multiply = [&](auto do_cut, const char* stage, uint4 (&r)[NJ][2], char* next_stage, const char* gnext) __attribute__((always_inline)) {
    constexpr bool CUT = decltype(do_cut)::value;
    static_for<SLOTS>([&](auto sc) __attribute__((always_inline)) {
      constexpr int S = decltype(sc)::value;
      constexpr int KB = S / (12 * NT), P = (S % (12 * NT)) / (2 * NT), t = (S % (2 * NT)) / 2, i = S % 2;
      if constexpr (S % (12 * NT) == 0) operands(stage, KB);
      mma_split_term<P>(acc[i][t], a3[i], b3[t]);
      if constexpr (CUT) {
        constexpr int U0 = S * CUT_UNITS / SLOTS, U1 = (S + 1) * CUT_UNITS / SLOTS;
        static_for<U1 - U0>([&](auto k) __attribute__((always_inline)) {
          cut_unit(std::integral_constant<int, U0 + decltype(k)::value>{}, r, next_stage, gnext);
        });
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  // Step s multiplies the pieces in stage s % 2 while the values of step s + 1 (asked for during step
  // s - 1) are cut into the other stage, row by row; each row's registers then ask for step s + 3.
  // Nothing in a step
  // is conditional (past the end the registers ask for the last step again, and the last step, which
  // has nothing to cut, stands alone after the loop): the waits the compiler places before the first
  // use of a value then leave the younger set of loads in flight.  Two steps per turn, so that each
  // register set keeps its role.
  const int last = steps - 1;
  fetch(raw[0], 0);
  fetch(raw[1], min(1, last));
  cut(raw[0], lds);
  fetch(raw[0], min(2, last));
  __syncthreads();
  auto step = [&](auto parity, int s) __attribute__((always_inline)) {
    constexpr int CUR = decltype(parity)::value;
    multiply(std::true_type{}, lds + CUR * STAGE, raw[CUR ^ 1], lds + (CUR ^ 1) * STAGE,
             step_base(min(s + 3, last)));
    __syncthreads();
  };
  int s = 0;
  for (; s + 2 < steps; s += 2) {
    step(std::integral_constant<int, 0>{}, s);
    step(std::integral_constant<int, 1>{}, s + 1);
  }
  if (s + 2 == steps) {
    step(std::integral_constant<int, 0>{}, s);
    multiply(std::false_type{}, lds + STAGE, raw[0], lds, xb);
  } else {
    multiply(std::false_type{}, lds, raw[1], lds + STAGE, xb);
  }
  __syncthreads();

  // squared norms: the four threads of a row add up their shares
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    float v = ss[j].total();
    v += __shfl_xor(v, 1);
    v += __shfl_xor(v, 2);
    const int row = lr + 64 * j;
    if (g4 == 0) {
      if (row < SIM_BM) norm2[row] = v;
      else normk[row - SIM_BM] = v;
    }
  }
  if (ANCHORED) {
    if (tid < SIM_BM) srow[tid] = s_hat[(int64_t)b * V + pruned[(int64_t)b * M + min(m0 + tid, M - 1)]];
  }
  __syncthreads();

  SimTile tile;
  tile.b = b; tile.B = B; tile.M = M; tile.k = k; tile.V = V; tile.m0 = m0; tile.n0 = n0; tile.pass = pass;
  tile.ptiles = ptiles; tile.mt = mt; tile.ks = ks; tile.ksplit = ksplit; tile.threshold = threshold;
  tile.kept = kept; tile.s_hat = s_hat; tile.assign = assign; tile.best_sim = best_sim; tile.best_key = best_key;
  tile.src_norm2 = src_norm2; tile.dots = dots; tile.kept_norm2 = kept_norm2;
  sim_tile_epilogue<NT, ANCHORED>(acc, norm2, normk, part, srow, tile);
}

// grid (ceil(n / 256)): the largest key over the destination tiles of a row -> assign, best_sim
__global__ __launch_bounds__(256) void k_sim_finish(const unsigned long long* __restrict__ best_key,
                                                     const float* __restrict__ src_norm2, int n, int ptiles,
                                                     float threshold, int32_t* __restrict__ assign,
                                                     float* __restrict__ best_sim) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  unsigned long long key = best_key[i];
  for (int t = 1; t < ptiles; ++t) {
    const unsigned long long other = best_key[(int64_t)t * n + i];
    key = other > key ? other : key;
  }
  const float v = float_unkey((uint32_t)(key >> 32));
  const int col = (int)(0xFFFFFFFFu - (uint32_t)key);
  const float c = v / fmaxf(sqrtf(src_norm2[i]), 1e-8f);
  best_sim[i] = c;
  assign[i] = (c > threshold) ? col : -1;
}

// grid (ceil(M / 4), B), 256 threads: one wave per source row.  Adds the ksplit partial products of
// every destination column in slice order, scales by the destination's norm, applies the predicate
// of the anchored search, takes the row's arg-max (ties to the smaller column) and divides by the
// source norm -- the arithmetic of k_sim's own epilogue.
template <bool ANCHORED>
__global__ __launch_bounds__(256) void k_sim_reduce(const float* __restrict__ dots, const float* __restrict__ src_norm2,
                                                     const float* __restrict__ kept_norm2, int B, int M, int k,
                                                     int ksplit, const int32_t* __restrict__ srcs,
                                                     const int32_t* __restrict__ kept, const float* __restrict__ s_hat,
                                                     int V, float threshold, int32_t* __restrict__ assign,
                                                     float* __restrict__ best_sim) {
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6), b = blockIdx.y;
  if (row >= M) return;
  const float sr_ = ANCHORED ? s_hat[(int64_t)b * V + srcs[(int64_t)b * M + row]] : 0.0f;
  float bv = -INFINITY;
  int bc = 0x7fffffff;
  for (int col = lane; col < k; col += 64) {
    // four running sums (slices q, q+1, q+2, q+3 of every four), so that the loads do not wait for
    // one another; the order of the additions is fixed all the same
    float d4[4] = {0.0f, 0.0f, 0.0f, 0.0f}, n4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    const int64_t dstride = (int64_t)B * M * k, nstride = (int64_t)B * k;
    const float* dp = dots + ((int64_t)b * M + row) * k + col;
    const float* np = kept_norm2 + (int64_t)b * k + col;
    int q = 0;
    for (; q + 3 < ksplit; q += 4) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        d4[u] += dp[(q + u) * dstride];
        n4[u] += np[(q + u) * nstride];
      }
    }
    for (; q < ksplit; ++q) {
      d4[0] += dp[q * dstride];
      n4[0] += np[q * nstride];
    }
    const float dot = (d4[0] + d4[1]) + (d4[2] + d4[3]), kn = (n4[0] + n4[1]) + (n4[2] + n4[3]);
    float c = dot * (1.0f / fmaxf(sqrtf(kn), 1e-8f));
    if (ANCHORED) {
      const float sc = s_hat[(int64_t)b * V + kept[(int64_t)b * k + col]];
      const bool stronger = (sc > sr_) | ((sc == sr_) & (col < row));
      c = stronger ? c : -INFINITY;
    }
    if (c > bv) { bv = c; bc = col; }             // a lane's columns ascend: the first maximum stays
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float ov = __shfl_xor(bv, off);
    const int oc = __shfl_xor(bc, off);
    if (ov > bv || (ov == bv && oc < bc)) { bv = ov; bc = oc; }
  }
  if (lane == 0) {
    float sn = 0.0f;
    for (int q = 0; q < ksplit; ++q) sn += src_norm2[((int64_t)q * B + b) * M + row];
    const float c = bv / fmaxf(sqrtf(sn), 1e-8f);
    best_sim[(int64_t)b * M + row] = c;
    assign[(int64_t)b * M + row] = (c > threshold) ? bc : -1;
  }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
static int pick_nt(const asap_params& p, int M);

// Slices of the hidden dimension: 1 unless the launch has at most 128 workgroups; then as many as
// bring it to about one workgroup per compute unit, with at least 8 steps per slice and a count that
// divides the steps, while the partial products stay under 64 MB.
static int pick_ksplit(const asap_params& p, int M, int nt) {
  const int bn = 64 * nt, ptiles = (p.k + bn - 1) / bn, mtiles = (M + SIM_BM - 1) / SIM_BM;
  const long wgs = (long)p.B * mtiles * ptiles;
  const int steps = p.D * (p.h_dtype == ASAP_BF16 ? 2 : 4) / SIM_ROWB;
  if (wgs > 128 || steps < 16) return 1;
  int ks = (int)(256 / wgs);
  if (ks > steps / 8) ks = steps / 8;
  while (ks > 1 && (steps % ks != 0 || (size_t)ks * p.B * M * p.k * sizeof(float) > ((size_t)64 << 20))) --ks;
  return ks < 1 ? 1 : ks;
}

// One key per destination tile and source row, and the source norms, for either kind of search
// (pruned -> kept: V-k source rows; inside the kept set: k), when the destination rows are split
// over several workgroups.
static size_t sim_workspace_for(const asap_params& p, int M) {
  if (M <= 0) return 0;
  const int nt = pick_nt(p, M), bn = 64 * nt, ptiles = (p.k + bn - 1) / bn, ks = pick_ksplit(p, M, nt);
  const size_t rows = (size_t)p.B * M;
  if (ks > 1)      // partial products, source norms, destination norms per slice
    return align256(sizeof(float) * ks * rows * p.k) + align256(sizeof(float) * ks * rows) +
           align256(sizeof(float) * ks * (size_t)p.B * p.k);
  return align256(sizeof(unsigned long long) * rows * ptiles) + align256(sizeof(float) * rows);
}
size_t sim_workspace_bytes(const asap_params& p) {
  const size_t a = sim_workspace_for(p, p.V - p.k), b = sim_workspace_for(p, p.k);
  return a > b ? a : b;
}

template <typename T, int NT, bool ANCHORED>
static hipError_t launch_sim_nt(const asap_params& p, const T* xv, int64_t sb, int64_t sr, const int32_t* srcs,
                                int M, const int32_t* kept, const float* s_hat, int32_t* assign, float* best_sim,
                                char* ws, hipStream_t st, Timer* tm) {
  constexpr int BN = 64 * NT;
  constexpr bool F32 = sizeof(T) == 4;
  static_assert(!F32 || NT <= SIMF_MAX_NT, "two steps of f32 pieces must fit LDS");
  const size_t lds = F32 ? (size_t)2 * (SIM_BM + BN) * SIMF_ROWP
                         : (size_t)(sim_na(NT) * SIM_BM + sim_nb(NT) * BN) * SIM_ROWB + sizeof(float) * (6 * SIM_BM + BN);
  auto kern = [] {
    if constexpr (F32) return k_sim_f32<NT, ANCHORED>;
    else return k_sim<T, NT, ANCHORED>;
  }();
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  const int mtiles = (M + SIM_BM - 1) / SIM_BM;
  const int ptiles = (p.k + BN - 1) / BN;
  const int spread = p.B >= NUM_XCD ? 1 : NUM_XCD / p.B;      // XCDs that share one image's source tiles
  const int vmt = (mtiles + spread - 1) / spread;
  const int groups = (p.B * spread + NUM_XCD - 1) / NUM_XCD;
  const int n = p.B * M;
  const int ksplit = pick_ksplit(p, M, NT);
  const char* label = F32 ? "k_sim_f32" : "k_sim";
  if (ksplit > 1) {
    float* dots = reinterpret_cast<float*>(ws);                                       // [ksplit][B][M][k]
    float* nsrc = reinterpret_cast<float*>(ws + align256(sizeof(float) * ksplit * (size_t)n * p.k));
    float* nkept = reinterpret_cast<float*>(reinterpret_cast<char*>(nsrc) + align256(sizeof(float) * ksplit * (size_t)n));
    ASAP_LAUNCH(tm, label, kern, dim3(NUM_XCD * groups * vmt * ptiles * ksplit), dim3(256), lds, st, xv, sb, sr, p.D,
                srcs, kept, s_hat, p.V, p.B, M, p.k, mtiles, ptiles, spread, vmt, p.sim_threshold, assign, best_sim,
                static_cast<unsigned long long*>(nullptr), nsrc, ksplit, dots, nkept);
    ASAP_LAUNCH(tm, "k_sim_reduce", k_sim_reduce<ANCHORED>, dim3((M + 3) / 4, p.B), dim3(256), 0, st, dots, nsrc, nkept,
                p.B, M, p.k, ksplit, srcs, kept, s_hat, p.V, p.sim_threshold, assign, best_sim);
    return hipGetLastError();
  }
  unsigned long long* keys = reinterpret_cast<unsigned long long*>(ws);               // [ptiles][B*M]
  float* norms = reinterpret_cast<float*>(ws + align256(sizeof(unsigned long long) * (size_t)n * ptiles));
  ASAP_LAUNCH(tm, label, kern, dim3(NUM_XCD * groups * vmt * ptiles), dim3(256), lds, st, xv, sb, sr, p.D, srcs,
              kept, s_hat, p.V, p.B, M, p.k, mtiles, ptiles, spread, vmt, p.sim_threshold, assign, best_sim, keys,
              norms, 1, static_cast<float*>(nullptr), static_cast<float*>(nullptr));
  if (ptiles > 1)
    ASAP_LAUNCH(tm, "k_sim_finish", k_sim_finish, dim3((n + 255) / 256), dim3(256), 0, st, keys, norms, n, ptiles,
                p.sim_threshold, assign, best_sim);
  return hipGetLastError();
}

// Destination tile width 64 * nt.  The kernel is bound by what a workgroup loads (or, for fp32, by
// what it multiplies): (128 + 64 nt) rows per step, over the steps of its slice of the hidden
// dimension, and the workgroups run in rounds of one per compute unit: fewest rounds x steps x rows
// (the slicing of pick_ksplit taken into account), then the wider tile.
static int pick_nt(const asap_params& p, int M) {
  const long mt = (M + SIM_BM - 1) / SIM_BM;
  const long steps = p.D * (p.h_dtype == ASAP_BF16 ? 2 : 4) / SIM_ROWB;
  const int nt_max = p.h_dtype == ASAP_BF16 ? 5 : SIMF_MAX_NT;
  int best_nt = nt_max;
  long best_cost = -1;
  for (int nt = nt_max; nt >= 1; --nt) {
    const long bn = 64 * nt, passes = (p.k + bn - 1) / bn;
    const long ks = pick_ksplit(p, M, nt);
    const long wgs = (long)p.B * mt * passes * ks, rounds = (wgs + 255) / 256;
    // a split launch also pays for the partial products' round trip and for k_sim_reduce: about as
    // much as 6000 row-steps, from measurements on the small configurations
    const long cost = rounds * (steps / ks) * (SIM_BM + bn) + (ks > 1 ? 6000 : 0);
    if (best_cost < 0 || cost < best_cost) { best_cost = cost; best_nt = nt; }
  }
  return best_nt;
}

template <typename T, bool ANCHORED>
static hipError_t sim_typed(const asap_params& p, const void* hidden, int64_t hsb, int64_t hsr,
                            const int32_t* kept, const int32_t* srcs, int M, const float* s_hat, int32_t* assign,
                            float* best_sim, char* ws, hipStream_t st, Timer* tm) {
  const T* xv = static_cast<const T*>(hidden) + (int64_t)p.P * hsr;
  switch (pick_nt(p, M)) {
    case 1: return launch_sim_nt<T, 1, ANCHORED>(p, xv, hsb, hsr, srcs, M, kept, s_hat, assign, best_sim, ws, st, tm);
    case 2: return launch_sim_nt<T, 2, ANCHORED>(p, xv, hsb, hsr, srcs, M, kept, s_hat, assign, best_sim, ws, st, tm);
    case 3: return launch_sim_nt<T, 3, ANCHORED>(p, xv, hsb, hsr, srcs, M, kept, s_hat, assign, best_sim, ws, st, tm);
    case 4: return launch_sim_nt<T, 4, ANCHORED>(p, xv, hsb, hsr, srcs, M, kept, s_hat, assign, best_sim, ws, st, tm);
    default:
      if constexpr (sizeof(T) == 2)
        return launch_sim_nt<T, 5, ANCHORED>(p, xv, hsb, hsr, srcs, M, kept, s_hat, assign, best_sim, ws, st, tm);
      else
        return hipErrorInvalidValue;        // pick_nt stays below for f32
  }
}

hipError_t launch_similarity(const asap_params& p, const void* hidden, int64_t hsb, int64_t hsr,
                             const int32_t* kept, const int32_t* srcs, int M, bool anchored, const float* s_hat,
                             int32_t* assign, float* best_sim, char* ws, hipStream_t st, Timer* tm) {
  const bool bf = p.h_dtype == ASAP_BF16;
  if (anchored)
    return bf ? sim_typed<bf16_t, true>(p, hidden, hsb, hsr, kept, srcs, M, s_hat, assign, best_sim, ws, st, tm)
              : sim_typed<float, true>(p, hidden, hsb, hsr, kept, srcs, M, s_hat, assign, best_sim, ws, st, tm);
  return bf ? sim_typed<bf16_t, false>(p, hidden, hsb, hsr, kept, srcs, M, s_hat, assign, best_sim, ws, st, tm)
            : sim_typed<float, false>(p, hidden, hsb, hsr, kept, srcs, M, s_hat, assign, best_sim, ws, st, tm);
}

}  // namespace asap
