// asap_select: the k largest scores of each image, ties to the smaller index, emitted as two
// ascending index lists.  One 1024-thread workgroup per image; everything stays in registers
// and LDS: a 4-pass, 8-bit radix search finds the k-th largest key, two block scans then place
// every index in its list.  Integer work throughout: the result is exact.
#include "asap_device.hpp"
#include "asap_launch.hpp"

namespace asap {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_IPT = 16;   // V <= 16384

// order-preserving map float -> uint32 (larger float, larger key)
__device__ __forceinline__ uint32_t float_key(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// exclusive block scan of one int per thread; returns the exclusive prefix, total via *total.
__device__ __forceinline__ int block_scan_excl(int x, int* wave_sums /*[17]*/, int* total) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int incl = x;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    int y = __shfl_up(incl, off);
    if (lane >= off) incl += y;
  }
  __syncthreads();                       // protects wave_sums against the previous use
  if (lane == 63) wave_sums[wave] = incl;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < SEL_THREADS / 64; ++w) {
    int s = wave_sums[w];
    if (w < wave) base += s;
    tot += s;
  }
  *total = tot;
  return base + incl - x;
}

__global__ __launch_bounds__(SEL_THREADS) void k_select(const float* __restrict__ score, int V, int k,
                                                         int32_t* __restrict__ kept, int32_t* __restrict__ pruned) {
  __shared__ int hist[512];   // two 256-bin histograms used alternately
  __shared__ int wave_sums[17];
  __shared__ int sel_bin, sel_remaining;
  const int b = blockIdx.x, tid = threadIdx.x;
  const float* sc = score + (int64_t)b * V;
  const int ipt = (V + SEL_THREADS - 1) / SEL_THREADS;      // items per thread, blocked layout
  const int i0 = tid * ipt;
  uint32_t key[SEL_IPT];
#pragma unroll
  for (int e = 0; e < SEL_IPT; ++e) {
    int i = i0 + e;
    key[e] = (e < ipt && i < V) ? float_key(sc[i]) : 0u;
  }

  uint32_t prefix = 0, mask = 0;
  int remaining = k;
  if (tid < 512) hist[tid] = 0;
  __syncthreads();
  for (int pass = 3; pass >= 0; --pass) {
    const int shift = 8 * pass;
    int* hcur = hist + (pass & 1) * 256;
#pragma unroll
    for (int e = 0; e < SEL_IPT; ++e) {
      int i = i0 + e;
      if (e < ipt && i < V && (key[e] & mask) == prefix) atomicAdd(&hcur[(key[e] >> shift) & 255u], 1);
    }
    __syncthreads();
    if (tid < 64) {
      // one wave walks the digits from 255 down: lane l holds digits 255-4l .. 252-4l
      int c[4], incl[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) c[q] = hcur[255 - (4 * tid + q)];
      incl[0] = c[0]; incl[1] = incl[0] + c[1]; incl[2] = incl[1] + c[2]; incl[3] = incl[2] + c[3];
      int run = incl[3];
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        int y = __shfl_up(run, off);
        if (tid >= off) run += y;
      }
      const int before = run - incl[3];         // candidates with a digit above this lane's four
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int upto = before + incl[q], above = upto - c[q];
        if (upto >= remaining && above < remaining) {
          sel_bin = 255 - (4 * tid + q);
          sel_remaining = remaining - above;
        }
      }
    } else if (tid >= 256 && tid < 512) {
      hist[((pass + 1) & 1) * 256 + (tid - 256)] = 0;    // the other histogram, for the next pass
    }
    __syncthreads();
    prefix |= (uint32_t)sel_bin << shift;
    mask |= 255u << shift;
    remaining = sel_remaining;
  }
  // prefix = the k-th largest key; `remaining` of the keys equal to it are kept, smallest index first
  const uint32_t thr = prefix;
  int n_eq = 0;
#pragma unroll
  for (int e = 0; e < SEL_IPT; ++e) {
    int i = i0 + e;
    if (e < ipt && i < V && key[e] == thr) ++n_eq;
  }
  int tot;
  int eq_before = block_scan_excl(n_eq, wave_sums, &tot);
  uint32_t keep_bits = 0;
  int n_keep = 0;
#pragma unroll
  for (int e = 0; e < SEL_IPT; ++e) {
    int i = i0 + e;
    if (e < ipt && i < V) {
      bool keep = key[e] > thr;
      if (key[e] == thr) { keep = eq_before < remaining; ++eq_before; }
      if (keep) { keep_bits |= 1u << e; ++n_keep; }
    }
  }
  int kept_before = block_scan_excl(n_keep, wave_sums, &tot);
  int32_t* kout = kept + (int64_t)b * k;
  int32_t* pout = pruned + (int64_t)b * (V - k);
#pragma unroll
  for (int e = 0; e < SEL_IPT; ++e) {
    int i = i0 + e;
    if (e < ipt && i < V) {
      if (keep_bits & (1u << e)) kout[kept_before++] = i;
      else pout[i - kept_before] = i;
    }
  }
}

hipError_t launch_select(const asap_params& p, const float* score, int32_t* kept, int32_t* pruned,
                         hipStream_t st, Timer* tm) {
  ASAP_LAUNCH(tm, "k_select", k_select, dim3(p.B), dim3(SEL_THREADS), 0, st, score, p.V, p.k, kept, pruned);
  return hipGetLastError();
}

}  // namespace asap
