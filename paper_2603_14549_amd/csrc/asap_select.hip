// asap_select: the k largest scores of each image, ties to the smaller index, emitted as two
// ascending index lists.  One 1024-thread workgroup per image; everything stays in registers
// and LDS: a 4-pass, 8-bit radix search finds the k-th largest key, two block scans then place
// every index in its list.  Integer work throughout: the result is exact.
#include "asap_launch.hpp"
#include "asap_select.hpp"

namespace asap {

__global__ __launch_bounds__(SEL_THREADS) void k_select(const float* __restrict__ score, int V, int k,
                                                         int32_t* __restrict__ kept, int32_t* __restrict__ pruned) {
  __shared__ SelectShared sh;
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
  int n_keep;
  const uint32_t keep_bits = radix_topk(key, ipt, i0, V, k, sh, &n_keep);
  int tot;
  int kept_before = block_scan_excl(n_keep, sh.wave_sums, &tot);
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
