// Device-side helpers shared by the gfx950 kernels of the pruning stage.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>
#include <utility>
#include <stdint.h>

namespace asap {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

struct bf16_t { uint16_t bits; };   // storage type tag for bfloat16 tensors

template <typename T> struct elem;
template <> struct elem<float>  { static constexpr int per16 = 4; };   // elements in a 16-byte chunk
template <> struct elem<bf16_t> { static constexpr int per16 = 8; };

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// round-to-nearest-even float -> bf16 bits (NaN kept quiet)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// Unpack a 16-byte chunk into floats: 4 for f32 storage, 8 for bf16 storage.
template <typename T> __device__ __forceinline__ void unpack16(const uint4& c, float* out);
template <> __device__ __forceinline__ void unpack16<float>(const uint4& c, float* out) {
  out[0] = __uint_as_float(c.x); out[1] = __uint_as_float(c.y);
  out[2] = __uint_as_float(c.z); out[3] = __uint_as_float(c.w);
}
template <> __device__ __forceinline__ void unpack16<bf16_t>(const uint4& c, float* out) {
  out[0] = bf16_bits_to_f32(c.x & 0xffffu); out[1] = bf16_bits_to_f32(c.x >> 16);
  out[2] = bf16_bits_to_f32(c.y & 0xffffu); out[3] = bf16_bits_to_f32(c.y >> 16);
  out[4] = bf16_bits_to_f32(c.z & 0xffffu); out[5] = bf16_bits_to_f32(c.z >> 16);
  out[6] = bf16_bits_to_f32(c.w & 0xffffu); out[7] = bf16_bits_to_f32(c.w >> 16);
}

template <typename T> __device__ __forceinline__ uint4 pack16(const float* in);
template <> __device__ __forceinline__ uint4 pack16<float>(const float* in) {
  return make_uint4(__float_as_uint(in[0]), __float_as_uint(in[1]), __float_as_uint(in[2]),
                    __float_as_uint(in[3]));
}
template <> __device__ __forceinline__ uint4 pack16<bf16_t>(const float* in) {
  return make_uint4(f32_to_bf16_bits(in[0]) | (f32_to_bf16_bits(in[1]) << 16),
                    f32_to_bf16_bits(in[2]) | (f32_to_bf16_bits(in[3]) << 16),
                    f32_to_bf16_bits(in[4]) | (f32_to_bf16_bits(in[5]) << 16),
                    f32_to_bf16_bits(in[6]) | (f32_to_bf16_bits(in[7]) << 16));
}

// One 16-byte operand chunk per lane on each side -> 32x32 fp32 tile update on the matrix
// cores.  Lane l supplies row (A) / column (B) l%32 and the contraction slice picked by l/32;
// which slice of the contraction dimension a chunk holds is the caller's choice as long as the
// A and B chunks of one call agree.  The 16 results of lane l are C[8*(v/4) + 4*(l/32) + v%4][l%32].
template <typename T> __device__ __forceinline__ void mma32(f32x16_t& acc, const uint4& a, const uint4& b);
template <> __device__ __forceinline__ void mma32<bf16_t>(f32x16_t& acc, const uint4& a, const uint4& b) {
  bf16x8_t x, y;
  __builtin_memcpy(&x, &a, 16);
  __builtin_memcpy(&y, &b, 16);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, acc, 0, 0, 0);
}
template <> __device__ __forceinline__ void mma32<float>(f32x16_t& acc, const uint4& a, const uint4& b) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
}

// ------------------------------------------------------------------------------------------
// Eight consecutive f32 values (two 16-byte chunks) as three bf16x8 operands: hi = rne(x),
// mid = rne(x - hi), lo = rne(x - hi - mid); the differences are exact, |x - hi - mid - lo| <= 2^-27 |x|.
// ------------------------------------------------------------------------------------------
typedef __bf16 sc_bf16x2 __attribute__((ext_vector_type(2)));
typedef float sc_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_bf16(float a, float b) {
  sc_f32x2 x = {a, b};
  sc_bf16x2 y = __builtin_convertvector(x, sc_bf16x2);
  uint32_t u;
  __builtin_memcpy(&u, &y, 4);
  return u;
}
struct Split3 { uint4 hi, mid, lo; };
__device__ __forceinline__ void split_pair(float a, float b, uint32_t& hi, uint32_t& mid, uint32_t& lo) {
  hi = pk_bf16(a, b);
  const float ra = a - __uint_as_float(hi << 16), rb = b - __uint_as_float(hi & 0xffff0000u);
  mid = pk_bf16(ra, rb);
  lo = pk_bf16(ra - __uint_as_float(mid << 16), rb - __uint_as_float(mid & 0xffff0000u));
}
__device__ __forceinline__ Split3 split_f32x8(const uint4& c0, const uint4& c1) {
  Split3 s;
  split_pair(__uint_as_float(c0.x), __uint_as_float(c0.y), s.hi.x, s.mid.x, s.lo.x);
  split_pair(__uint_as_float(c0.z), __uint_as_float(c0.w), s.hi.y, s.mid.y, s.lo.y);
  split_pair(__uint_as_float(c1.x), __uint_as_float(c1.y), s.hi.z, s.mid.z, s.lo.z);
  split_pair(__uint_as_float(c1.z), __uint_as_float(c1.w), s.hi.w, s.mid.w, s.lo.w);
  return s;
}
// The six piece products of one contraction group, smallest first, into one accumulator: the small
// ones land on partial sums of the large ones, i.e. they are rounded at the level the hi.hi products
// of the row are rounded at anyway (2^-24 of the running sum).
__device__ __forceinline__ void mma_split(f32x16_t& acc, const Split3& a, const Split3& b) {
  mma32<bf16_t>(acc, a.lo, b.hi);
  mma32<bf16_t>(acc, a.hi, b.lo);
  mma32<bf16_t>(acc, a.mid, b.mid);
  mma32<bf16_t>(acc, a.mid, b.hi);
  mma32<bf16_t>(acc, a.hi, b.mid);
  mma32<bf16_t>(acc, a.hi, b.hi);
}

// The same products one at a time: product P (0..5, in the order of mma_split) of a group.  A caller
// that walks P in its outer loop and the accumulators in its inner loop adds the same terms in the same
// order per accumulator, with independent matrix instructions next to each other.
template <int P> __device__ __forceinline__ void mma_split_term(f32x16_t& acc, const Split3& a, const Split3& b) {
  static_assert(P >= 0 && P < 6, "six piece products");
  if constexpr (P == 0) mma32<bf16_t>(acc, a.lo, b.hi);
  else if constexpr (P == 1) mma32<bf16_t>(acc, a.hi, b.lo);
  else if constexpr (P == 2) mma32<bf16_t>(acc, a.mid, b.mid);
  else if constexpr (P == 3) mma32<bf16_t>(acc, a.mid, b.hi);
  else if constexpr (P == 4) mma32<bf16_t>(acc, a.hi, b.mid);
  else mma32<bf16_t>(acc, a.hi, b.hi);
}

// row of the 32x32 tile held in accumulator register v of lane l
__device__ __forceinline__ int mma32_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

__device__ __forceinline__ double shfl_xor_f64(double x, int mask) {
  int lo = __double2loint(x), hi = __double2hiint(x);
  lo = __shfl_xor(lo, mask);
  hi = __shfl_xor(hi, mask);
  return __hiloint2double(hi, lo);
}

__device__ __forceinline__ uint4 ldg16(const void* p) { return *reinterpret_cast<const uint4*>(p); }

// 16-byte load of data that is read exactly once: marked non-temporal so that it does not push
// out of the caches what later kernels come back to.
typedef uint32_t u32x4_nt __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ldg16_stream(const void* p) {
  u32x4_nt x = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt*>(p));
  return make_uint4(x.x, x.y, x.z, x.w);
}

// 16-byte store of data this stage does not read again (outputs): marked non-temporal so that the
// lines do not linger dirty in the caches and get written back under a later kernel's reads.
__device__ __forceinline__ void stg16_stream(void* p, const uint4& v) {
  u32x4_nt x = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(x, reinterpret_cast<u32x4_nt*>(p));
}

// ------------------------------------------------------------------------------------------
// direct global -> LDS loads and the hand-placed waits that go with them
// ------------------------------------------------------------------------------------------
// m0 is named as clobbered by the load helper below on purpose
#pragma clang diagnostic ignored "-Winline-asm"

// 16 bytes per lane from global memory straight into LDS: lane L's data, read from gbase + voff
// (gbase wave-uniform), lands at LDS byte address lds_addr + 16 L (lds_addr wave-uniform, passed
// in M0).  Completion is counted by vmcnt.  Written as assembly so that the compiler does not
// order the workgroup's own LDS operand reads behind every outstanding load (it cannot tell the
// ring slots apart); the waits below are placed by hand instead.
__device__ __forceinline__ void load_to_lds16(const char* gbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(voff), "s"(gbase), "s"(lds_addr) : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_address(const void* p) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}
__device__ __forceinline__ void wait_all_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// wait until at most N (< 64) of this wave's vector-memory loads are still outstanding
template <int N> __device__ __forceinline__ void wait_vmem_but() {
  static_assert(N >= 0 && N < 64, "vmcnt field");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// Workgroup barrier without the release fence of __syncthreads(): that fence would wait for every
// outstanding load of the wave, also the ones that are meant to stay in flight across the barrier.
__device__ __forceinline__ void barrier_keep_loads() { asm volatile("s_barrier" ::: "memory"); }

// f(integral_constant<int, 0>), ..., f(integral_constant<int, N - 1>): a loop whose counter is a
// compile-time constant inside the body
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

}  // namespace asap
