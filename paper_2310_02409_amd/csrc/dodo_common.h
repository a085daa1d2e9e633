// Internal helpers shared by the HIP translation units of libdodo (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dodo.h"

namespace dodo {

constexpr int kWave = 64;

// Records the HIP error text for dodo_status_string and maps it to DODO_ERR_HIP.
int record_hip_error(hipError_t e);

#define DODO_HIP_TRY(expr)                                      \
  do {                                                          \
    hipError_t e_ = (expr);                                     \
    if (e_ != hipSuccess) return ::dodo::record_hip_error(e_);  \
  } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int elem_bytes(int dtype) { return dtype == DODO_DTYPE_F32 ? 4 : 2; }
inline bool dtype_ok(int dtype) { return dtype == DODO_DTYPE_F32 || dtype == DODO_DTYPE_BF16; }

// Compute units of the current device (256 if the query fails); asked once per device, then remembered.
int compute_units();

// Makes sure `kernel` may be launched with `bytes` of dynamic LDS on the current device.  The runtime is asked
// only when a kernel needs more than it was granted before on that device, so the launch path stays free of it.
int allow_dynamic_lds(const void* kernel, int bytes);

// Workgroups of `kernel` (with `threads` threads and `lds` bytes of dynamic LDS) that a compute unit of the
// current device holds at once; asked once per (device, kernel, lds), then remembered.  `fallback` if the query fails.
int resident_blocks_per_cu(const void* kernel, int threads, size_t lds, int fallback);

// Checks the launch that was just enqueued.
inline int launch_status() {
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DODO_OK : record_hip_error(e);
}

// bf16 <-> fp32 on raw bits (bf16 is the upper half of an fp32).
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }
// round-to-nearest-even fp32 -> bf16 bits (NaN kept quiet)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// 16-byte global load / store with the non-temporal hint (streamed once, no reuse)
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load16_stream(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load(static_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store16_stream(void* p, const uint4& v) {
  u32x4_t t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, static_cast<u32x4_t*>(p));
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// Order-preserving image of an fp32 score as an unsigned key: NaN ranks below everything, -0 == +0.
__device__ __forceinline__ uint32_t order_key(float s) {
  uint32_t u = __float_as_uint(s);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Element i of an fp32 or bf16 array as fp32.
template <int DTYPE>
__device__ __forceinline__ float load_elem(const void* p, int64_t i) {
  if (DTYPE == DODO_DTYPE_F32) return static_cast<const float*>(p)[i];
  return __uint_as_float(static_cast<uint32_t>(static_cast<const uint16_t*>(p)[i]) << 16);
}

// One 16-byte-per-lane direct global->LDS load from base + voff: the lanes' data land at lds_dst + 16*lane; base
// and lds_dst are wavefront-uniform (base is made so explicitly: the compiler may hold it in vector registers).
// Inline assembly, so the compiler does not order later LDS reads behind it: callers keep the vmcnt bookkeeping.
__device__ __forceinline__ void dma16_uniform(const void* base, uint32_t voff, uint32_t lds_dst) {
  const uint64_t b = reinterpret_cast<uint64_t>(base);
  const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(b))));
  const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(b >> 32))));
  const uint64_t ub = (static_cast<uint64_t>(hi) << 32) | static_cast<uint64_t>(lo);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(ub), "s"(lds_dst)
               : "memory", "m0");
}

// Sum over groups of NL consecutive lanes (NL = 8 or 16: inside one row of 16 lanes), every lane getting its
// group's total: data-parallel-primitive adds with the partner lane of a pair, the partner pair of a quad, the
// mirrored half and the mirrored row.  At every step the partner holds its own group's sum in all of its lanes and
// both sides add the same two numbers, so all lanes of a group end with the same bits.  No LDS traffic.
template <int NL>
__device__ __forceinline__ float lanes_sum(float x) {
  static_assert(NL == 8 || NL == 16, "groups of 8 or 16 lanes");
#define DODO_DPP_ADD(CTRL) \
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false))
  DODO_DPP_ADD(0xB1);                // quad_perm [1,0,3,2]
  DODO_DPP_ADD(0x4E);                // quad_perm [2,3,0,1]
  DODO_DPP_ADD(0x141);               // row_half_mirror: lane i <-> 7 - i of each 8
  if (NL == 16) DODO_DPP_ADD(0x140);  // row_mirror: lane i <-> 15 - i
#undef DODO_DPP_ADD
  return x;
}
// Sum over the 64 lanes of a wavefront, the same bits in every lane: the four rows' sums, read as scalars.
__device__ __forceinline__ float wave_sum64(float x) {
  const int r = __builtin_bit_cast(int, lanes_sum<16>(x));
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(r, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(r, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(r, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(r, 48));
  return (r0 + r1) + (r2 + r3);
}

// Division of a number below 2^31 by a divisor fixed on the host: one 32 x 32 -> 64 bit multiplication and a
// shift, which stay on the scalar unit for a wavefront-uniform dividend (a division by a run-time value would be
// some thirty vector instructions).  mul = ceil(2^shift / d), shift = 31 + ceil(log2 d): exact for all x < 2^31.
struct FastDiv {
  uint32_t mul, shift;
};
inline FastDiv make_fast_div(uint32_t d) {
  uint32_t l = 0;
  while ((1ull << l) < d) ++l;
  FastDiv f;
  f.shift = 31 + l;
  f.mul = static_cast<uint32_t>(((1ull << f.shift) + d - 1) / d);
  return f;
}
__device__ __forceinline__ uint32_t fast_div(uint32_t x, FastDiv f) {
  return static_cast<uint32_t>((static_cast<uint64_t>(x) * f.mul) >> f.shift);
}

// number of set bits of `mask` strictly below this lane
__device__ __forceinline__ int popc_below_lane(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
}

}  // namespace dodo
