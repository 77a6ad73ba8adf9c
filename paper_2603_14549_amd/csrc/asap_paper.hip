// Second half of the routing of Sec. 4.2 (ASAP_ROUTE_PAPER), after the anchored similarity search
// of asap_sim.hip has given every kept token its destination inside the kept set (or none):
//   * chains of destinations are followed to their roots, so that every tree merges into one token
//     that is not itself a source (a destination is strictly stronger than its source -- larger
//     salience, ties to the smaller index -- so there are no cycles);
//   * the a vacated slots are refilled with the a pruned tokens of largest raw attention mass s_j
//     (ties to the smaller index), which stay unmerged ("budget reallocation");
//   * the final kept list = roots and refills, ascending, and for every kept slot the slot (in the
//     final list) of the root that absorbs it, -1 if it survives.
//
//   k_paper_plan   one 1024-thread workgroup per image, everything in LDS; the refill reuses the
//                  exact radix selection of asap_select.  Integer work apart from the key map.
#include "asap_launch.hpp"
#include "asap_select.hpp"

namespace asap {

// slot_of[] states before the final positions are known
constexpr int TOK_PRUNED = -1, TOK_ROOT = -2, TOK_SOURCE = -3;

__global__ __launch_bounds__(SEL_THREADS) void k_paper_plan(const int32_t* __restrict__ dest,
                                                             const int32_t* __restrict__ kept,
                                                             const float* __restrict__ s_raw, int V, int k,
                                                             int32_t* __restrict__ final_idx,
                                                             int32_t* __restrict__ assign) {
  __shared__ SelectShared sh;
  extern __shared__ int32_t dyn[];
  int32_t* root = dyn;            // [k]  destination of a kept slot, then the root of its tree
  int32_t* slot_of = dyn + k;     // [V]  token state, then the slot of a final token
  const int b = blockIdx.x, tid = threadIdx.x;
  const int32_t* kp = kept + (int64_t)b * k;

  for (int a = tid; a < k; a += SEL_THREADS) root[a] = dest[(int64_t)b * k + a];
  for (int i = tid; i < V; i += SEL_THREADS) slot_of[i] = TOK_PRUNED;
  __syncthreads();
  // roots: at most k-1 hops (the bound only guards against a malformed destination list)
  constexpr int SPT = (SEL_IPT * SEL_THREADS / 2 + SEL_THREADS - 1) / SEL_THREADS;   // kept slots per thread, k <= V/2
  int rt[SPT];
  int n_src = 0;
#pragma unroll
  for (int e = 0; e < SPT; ++e) {
    const int a = tid + e * SEL_THREADS;
    rt[e] = a;
    if (a < k) {
      int r = a;
      for (int hop = 0; hop < k && root[r] >= 0; ++hop) r = root[r];
      rt[e] = r;
      n_src += (r != a);
    }
  }
  int n_vacated;
  block_scan_excl(n_src, sh.wave_sums, &n_vacated);      // its barriers also end the reads of root[]
#pragma unroll
  for (int e = 0; e < SPT; ++e) {
    const int a = tid + e * SEL_THREADS;
    if (a < k) {
      root[a] = rt[e];
      slot_of[kp[a]] = (rt[e] == a) ? TOK_ROOT : TOK_SOURCE;
    }
  }
  __syncthreads();

  // refill: the n_vacated largest s_raw among the pruned tokens
  const int ipt = (V + SEL_THREADS - 1) / SEL_THREADS;      // items per thread, blocked layout
  const int i0 = tid * ipt;
  uint32_t key[SEL_IPT];
#pragma unroll
  for (int e = 0; e < SEL_IPT; ++e) {
    const int i = i0 + e;
    key[e] = (e < ipt && i < V && slot_of[i] == TOK_PRUNED) ? float_key(s_raw[(int64_t)b * V + i]) : 0u;
  }
  int n_mine;
  const uint32_t refill = radix_topk(key, ipt, i0, V, n_vacated, sh, &n_mine);

  // final list, ascending
  int n_fin = 0;
  uint32_t fin = 0;
#pragma unroll
  for (int e = 0; e < SEL_IPT; ++e) {
    const int i = i0 + e;
    if (e < ipt && i < V && ((refill >> e & 1u) || slot_of[i] == TOK_ROOT)) { fin |= 1u << e; ++n_fin; }
  }
  int tot;
  int pos = block_scan_excl(n_fin, sh.wave_sums, &tot);
#pragma unroll
  for (int e = 0; e < SEL_IPT; ++e) {
    const int i = i0 + e;
    if (fin >> e & 1u) {
      if (pos < k) final_idx[(int64_t)b * k + pos] = i;
      slot_of[i] = pos++;
    }
  }
  __syncthreads();
  for (int a = tid; a < k; a += SEL_THREADS) {
    const int r = root[a];
    assign[(int64_t)b * k + a] = (r == a) ? -1 : slot_of[kp[r]];
  }
}

size_t paper_workspace_bytes(const asap_params& p) {
  // destinations [B,k] int32 of the anchored similarity search
  return p.route == ASAP_ROUTE_PAPER ? align256(sizeof(int32_t) * (size_t)p.B * p.k) : 0;
}

hipError_t launch_paper_plan(const asap_params& p, const int32_t* dest, const int32_t* kept, const float* s_raw,
                             int32_t* final_idx, int32_t* assign, hipStream_t st, Timer* tm) {
  const size_t lds = sizeof(int32_t) * ((size_t)p.k + p.V);
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_paper_plan),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  ASAP_LAUNCH(tm, "k_paper_plan", k_paper_plan, dim3(p.B), dim3(SEL_THREADS), lds, st, dest, kept, s_raw, p.V, p.k,
              final_idx, assign);
  return hipGetLastError();
}

}  // namespace asap
