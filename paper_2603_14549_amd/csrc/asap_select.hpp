// Exact top-k selection inside one 1024-thread workgroup, shared by the selection kernel and by the
// budget reallocation of the paper's routing: a 4-pass, 8-bit radix search finds the k-th largest
// key, a block scan then decides which of the keys equal to it are taken (smallest index first).
// Integer work throughout.
#pragma once
#include "asap_device.hpp"

namespace asap {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_IPT = 16;   // V <= 16384

// order-preserving map float -> uint32 (larger float, larger key); every finite float maps above 0
__device__ __forceinline__ uint32_t float_key(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float float_unkey(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
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

// LDS the selection needs
struct SelectShared {
  int hist[512];        // two 256-bin histograms used alternately
  int wave_sums[17];
  int sel_bin, sel_remaining;
};

// Thread tid holds the keys of items i0 .. i0+ipt-1 (blocked layout, so index order = thread order);
// items past V or not taking part carry key 0 and `take` must not exceed the number of keys > 0.
// Returns the bit mask of this thread's items among the `take` largest (ties: smaller index) and
// their count.  All threads of the workgroup must call it; take is the same for all.
__device__ __forceinline__ uint32_t radix_topk(const uint32_t (&key)[SEL_IPT], int ipt, int i0, int V, int take,
                                               SelectShared& sh, int* n_mine) {
  const int tid = threadIdx.x;
  *n_mine = 0;
  if (take <= 0) return 0u;
  uint32_t prefix = 0, mask = 0;
  int remaining = take;
  __syncthreads();                       // the histograms may still be read from an earlier call
  if (tid < 512) sh.hist[tid] = 0;
  __syncthreads();
  for (int pass = 3; pass >= 0; --pass) {
    const int shift = 8 * pass;
    int* hcur = sh.hist + (pass & 1) * 256;
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
          sh.sel_bin = 255 - (4 * tid + q);
          sh.sel_remaining = remaining - above;
        }
      }
    } else if (tid >= 256 && tid < 512) {
      sh.hist[((pass + 1) & 1) * 256 + (tid - 256)] = 0;    // the other histogram, for the next pass
    }
    __syncthreads();
    prefix |= (uint32_t)sh.sel_bin << shift;
    mask |= 255u << shift;
    remaining = sh.sel_remaining;
  }
  // prefix = the take-th largest key; `remaining` of the keys equal to it are taken, smallest index first
  const uint32_t thr = prefix;
  int n_eq = 0;
#pragma unroll
  for (int e = 0; e < SEL_IPT; ++e) {
    int i = i0 + e;
    if (e < ipt && i < V && key[e] == thr) ++n_eq;
  }
  int tot;
  int eq_before = block_scan_excl(n_eq, sh.wave_sums, &tot);
  uint32_t bits = 0;
  int n = 0;
#pragma unroll
  for (int e = 0; e < SEL_IPT; ++e) {
    int i = i0 + e;
    if (e < ipt && i < V) {
      bool keep = key[e] > thr;
      if (key[e] == thr) { keep = eq_before < remaining; ++eq_before; }
      if (keep) { bits |= 1u << e; ++n; }
    }
  }
  *n_mine = n;
  return bits;
}

}  // namespace asap
