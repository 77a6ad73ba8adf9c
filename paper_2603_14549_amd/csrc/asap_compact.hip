// asap_compact_kv: gathers the K/V rows of the surviving positions of every cached layer
// (KV-cache compatibility of the pruning stage).  Pure data movement, bit-exact.
//
// k_positions: grid (ceil(Nout / 256), B): the positions the compaction gathers, from the kept set alone.
// k_compact<MODE>: grid (ceil(rows / ROWS_PER_BLOCK), B * Hkv, 2 * layers_in_launch), 256 threads, rows = Nout
// or, for the kept tokens' rows alone, k; the source rows come from the position list or straight from the
// kept list (then nothing of asap_merge is needed).
// k_compact_paged: the same grid for caches kept as pools of pages with one block table per sequence.
// A row is d elements = LPR 16-byte pieces; LPR consecutive lanes move one row.
#include "asap_device.hpp"
#include "asap_launch.hpp"

namespace asap {

constexpr int KV_ROWS_PER_THREAD = 4;

void fill_kv_pointers(KvPointers* ptrs, int n_layers, const void* const* k_src, const void* const* v_src,
                      void* const* k_dst, void* const* v_dst) {
  for (int l = 0; l < n_layers; ++l) {
    ptrs->src[2 * l] = static_cast<const char*>(k_src[l]);
    ptrs->src[2 * l + 1] = static_cast<const char*>(v_src[l]);
    ptrs->dst[2 * l] = static_cast<char*>(k_dst[l]);
    ptrs->dst[2 * l + 1] = static_cast<char*>(v_dst[l]);
  }
  for (int l = 2 * n_layers; l < 2 * KV_LAYERS_PER_LAUNCH; ++l) { ptrs->src[l] = nullptr; ptrs->dst[l] = nullptr; }
}

// Where the source rows come from: the position list of asap_merge / asap_positions, or the kept list
// and text_len directly (the output order of Fig. 3 written out: prefix | kept | valid text).
// idx = pos_out [B,Nout] and len = new_len (BY_POS); idx = kept list [B,k] and len = text_len (FROM_KEPT,
// KEPT_ONLY); FIXED_ONLY reads no index list and takes len = text_len.
template <int MODE>
__device__ __forceinline__ void compact_block(const KvPointers& ptrs, const int32_t* __restrict__ idx,
                                              const int32_t* __restrict__ len, int Hkv, int N, int Nout,
                                              int row_bytes, int P, int V, int k, int bx, int bg, int bz) {
  const int lpr = row_bytes >> 4, rpi = 256 / lpr;
  const int tid = threadIdx.x, piece = tid % lpr, r0 = tid / lpr;
  const int b = bg / Hkv;
  const int n_rows = MODE == KV_BY_POS      ? min(len[b], Nout)
                     : MODE == KV_KEPT_ONLY ? k
                     : MODE == KV_FIXED_ONLY ? P + min(max(len[b], 0), Nout - P - k)
                                             : P + k + min(len[b], Nout - P - k);
  const char* src = ptrs.src[bz] + (int64_t)bg * N * row_bytes + piece * 16;
  char* dst = ptrs.dst[bz] + (int64_t)bg * Nout * row_bytes + piece * 16;
  const int32_t* ix = idx + (int64_t)b * (MODE == KV_BY_POS ? Nout : k);
  const int base = bx * rpi * KV_ROWS_PER_THREAD + r0;
  uint4 v[KV_ROWS_PER_THREAD];
#pragma unroll
  for (int i = 0; i < KV_ROWS_PER_THREAD; ++i) {
    const int r = base + i * rpi;
    if (r < n_rows) {
      const int srow = MODE == KV_BY_POS       ? ix[r]
                       : MODE == KV_KEPT_ONLY  ? P + ix[r]
                       : MODE == KV_FIXED_ONLY ? (r < P ? r : r + V)
                       : r < P                 ? r
                       : r < P + k             ? P + ix[r - P]
                                               : r - k + V;
      v[i] = ldg16_stream(src + (int64_t)srow * row_bytes);
    }
  }
#pragma unroll
  for (int i = 0; i < KV_ROWS_PER_THREAD; ++i) {
    const int r = base + i * rpi;
    // kept slot r is output row P + r; the r-th row that no selection changes is output row r (prefix) or
    // r + k (text)
    const int drow = MODE == KV_KEPT_ONLY ? P + r : MODE == KV_FIXED_ONLY ? (r < P ? r : r + k) : r;
    if (r < n_rows) stg16_stream(dst + (int64_t)drow * row_bytes, v[i]);
  }
}

template <int MODE>
__global__ __launch_bounds__(256) void k_compact(KvPointers ptrs, const int32_t* __restrict__ idx,
                                                  const int32_t* __restrict__ len, int Hkv, int N, int Nout,
                                                  int row_bytes, int P, int V, int k) {
  compact_block<MODE>(ptrs, idx, len, Hkv, N, Nout, row_bytes, P, V, k, blockIdx.x, blockIdx.y, blockIdx.z);
}

// The rows that no selection changes, for the launch that runs beside the score kernels: a grid of
// at most two workgroups per compute unit walks the (gx, gy, gz) blocks of k_compact, so that the
// kernels of the other stream still find room on every compute unit.
__global__ __launch_bounds__(256) void k_compact_fixed(KvPointers ptrs, const int32_t* __restrict__ len, int Hkv,
                                                        int N, int Nout, int row_bytes, int P, int V, int k, int gx,
                                                        int gy, int gz) {
  const int total = gx * gy * gz;
  for (int id = blockIdx.x; id < total; id += gridDim.x) {
    const int bx = id % gx, bg = (id / gx) % gy, bz = id / (gx * gy);
    compact_block<KV_FIXED_ONLY>(ptrs, len, len, Hkv, N, Nout, row_bytes, P, V, k, bx, bg, bz);
  }
}

// Pools are [n_pages, Hkv, page_size, d]; token n of sequence b is in page table[b, n / page_size],
// slot n % page_size.
__global__ __launch_bounds__(256) void k_compact_paged(KvPointers ptrs, const int32_t* __restrict__ pos_out,
                                                        const int32_t* __restrict__ new_len,
                                                        const int32_t* __restrict__ src_table, int src_stride,
                                                        const int32_t* __restrict__ dst_table, int dst_stride,
                                                        int page_size, int Hkv, int Nout, int row_bytes) {
  const int lpr = row_bytes >> 4, rpi = 256 / lpr;
  const int tid = threadIdx.x, piece = tid % lpr, r0 = tid / lpr;
  const int bg = blockIdx.y, b = bg / Hkv, g = bg % Hkv;
  const int nl = new_len[b];
  const char* src = ptrs.src[blockIdx.z] + piece * 16;
  char* dst = ptrs.dst[blockIdx.z] + piece * 16;
  const int32_t* pos = pos_out + (int64_t)b * Nout;
  const int32_t* stab = src_table + (int64_t)b * src_stride;
  const int32_t* dtab = dst_table + (int64_t)b * dst_stride;
  const int base = blockIdx.x * rpi * KV_ROWS_PER_THREAD + r0;
  uint4 v[KV_ROWS_PER_THREAD];
#pragma unroll
  for (int i = 0; i < KV_ROWS_PER_THREAD; ++i) {
    const int nrow = base + i * rpi;
    if (nrow < nl) {
      const int m = pos[nrow];
      const int64_t row = ((int64_t)stab[m / page_size] * Hkv + g) * page_size + m % page_size;
      v[i] = ldg16_stream(src + row * row_bytes);
    }
  }
#pragma unroll
  for (int i = 0; i < KV_ROWS_PER_THREAD; ++i) {
    const int nrow = base + i * rpi;
    if (nrow < nl) {
      const int64_t row = ((int64_t)dtab[nrow / page_size] * Hkv + g) * page_size + nrow % page_size;
      stg16_stream(dst + row * row_bytes, v[i]);
    }
  }
}

// Output order of the stage (Fig. 3, Sec. 4.2): prefix | kept tokens in original order | valid text.
__global__ __launch_bounds__(256) void k_positions(const int32_t* __restrict__ kept, const int32_t* __restrict__ text_len,
                                                    int P, int V, int k, int Nout, int32_t* __restrict__ pos_out,
                                                    int32_t* __restrict__ new_len) {
  const int b = blockIdx.y, n = blockIdx.x * 256 + threadIdx.x;
  const int len = text_len[b];
  if (n == 0) new_len[b] = P + k + len;
  if (n >= Nout) return;
  int pos;
  if (n < P) pos = n;
  else if (n < P + k) pos = P + kept[(int64_t)b * k + (n - P)];
  else pos = (n - P - k < len) ? P + V + (n - P - k) : -1;
  pos_out[(int64_t)b * Nout + n] = pos;
}

hipError_t launch_positions(const asap_params& p, const int32_t* kept, const int32_t* text_len, int32_t* pos_out,
                            int32_t* new_len, hipStream_t st, Timer* tm) {
  const int Nout = p.P + p.k + p.Tmax;
  ASAP_LAUNCH(tm, "k_positions", k_positions, dim3((Nout + 255) / 256, p.B), dim3(256), 0, st, kept, text_len, p.P,
              p.V, p.k, Nout, pos_out, new_len);
  return hipGetLastError();
}

// mode: KV_BY_POS (idx = pos_out, len = new_len) or KV_FROM_KEPT (idx = kept list, len = text_len)
hipError_t launch_compact_kv(const asap_params& p, int mode, int n_layers, const void* const* k_src,
                             const void* const* v_src, void* const* k_dst, void* const* v_dst,
                             const int32_t* idx, const int32_t* len, hipStream_t st, Timer* tm) {
  const int row_bytes = p.d * (p.kv_dtype == ASAP_BF16 ? 2 : 4);
  const int N = p.P + p.V + p.Tmax, Nout = p.P + p.k + p.Tmax;
  const int rows_per_block = (256 / (row_bytes / 16)) * KV_ROWS_PER_THREAD;
  const int rows = mode == KV_KEPT_ONLY ? p.k : mode == KV_FIXED_ONLY ? p.P + p.Tmax : Nout;
  for (int l0 = 0; l0 < n_layers; l0 += KV_LAYERS_PER_LAUNCH) {
    const int nl = n_layers - l0 < KV_LAYERS_PER_LAUNCH ? n_layers - l0 : KV_LAYERS_PER_LAUNCH;
    KvPointers ptrs;
    fill_kv_pointers(&ptrs, nl, k_src + l0, v_src + l0, k_dst + l0, v_dst + l0);
    dim3 grid((rows + rows_per_block - 1) / rows_per_block, p.B * p.Hkv, 2 * nl);
    if (mode == KV_BY_POS)
      ASAP_LAUNCH(tm, "k_compact", k_compact<KV_BY_POS>, grid, dim3(256), 0, st, ptrs, idx, len, p.Hkv, N, Nout,
                  row_bytes, p.P, p.V, p.k);
    else if (mode == KV_FROM_KEPT)
      ASAP_LAUNCH(tm, "k_compact", k_compact<KV_FROM_KEPT>, grid, dim3(256), 0, st, ptrs, idx, len, p.Hkv, N, Nout,
                  row_bytes, p.P, p.V, p.k);
    else if (mode == KV_KEPT_ONLY)
      ASAP_LAUNCH(tm, "k_compact", k_compact<KV_KEPT_ONLY>, grid, dim3(256), 0, st, ptrs, idx, len, p.Hkv, N, Nout,
                  row_bytes, p.P, p.V, p.k);
    else {
      const long total = (long)grid.x * grid.y * grid.z;
      ASAP_LAUNCH(tm, "k_compact_fixed", k_compact_fixed, dim3((unsigned)(total < 512 ? total : 512)), dim3(256), 0, st,
                  ptrs, len, p.Hkv, N, Nout, row_bytes, p.P, p.V, p.k, (int)grid.x, (int)grid.y, (int)grid.z);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_compact_kv_paged(const asap_params& p, int n_layers, const void* const* k_src,
                                   const void* const* v_src, void* const* k_dst, void* const* v_dst, int page_size,
                                   const int32_t* src_table, int src_stride, const int32_t* dst_table,
                                   int dst_stride, const int32_t* pos_out, const int32_t* new_len, hipStream_t st,
                                   Timer* tm) {
  const int row_bytes = p.d * (p.kv_dtype == ASAP_BF16 ? 2 : 4);
  const int Nout = p.P + p.k + p.Tmax;
  const int rows_per_block = (256 / (row_bytes / 16)) * KV_ROWS_PER_THREAD;
  for (int l0 = 0; l0 < n_layers; l0 += KV_LAYERS_PER_LAUNCH) {
    const int nl = n_layers - l0 < KV_LAYERS_PER_LAUNCH ? n_layers - l0 : KV_LAYERS_PER_LAUNCH;
    KvPointers ptrs;
    fill_kv_pointers(&ptrs, nl, k_src + l0, v_src + l0, k_dst + l0, v_dst + l0);
    dim3 grid((Nout + rows_per_block - 1) / rows_per_block, p.B * p.Hkv, 2 * nl);
    ASAP_LAUNCH(tm, "k_compact_paged", k_compact_paged, grid, dim3(256), 0, st, ptrs, pos_out, new_len, src_table,
                src_stride, dst_table, dst_stride, page_size, p.Hkv, Nout, row_bytes);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace asap
