// Device-side helpers shared by the LASER-KV kernels (gfx950 / CDNA4, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lkv {

constexpr int DT_F32 = 0;
constexpr int DT_BF16 = 1;

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr float NEG_BIG = -1.0e30f;  // finite stand-in for -inf (keeps max/sub free of NaN)

// One 32x32 MFMA tile step over a 16-byte operand chunk per lane.
//
// Operand convention used by every kernel here: lane l = (rl, kg) with rl = l & 31 the
// row (of A) / column (of B) inside the 32-wide tile and kg = l >> 5 the half of the
// contraction slice the lane feeds.  For chunk-pair index i a lane loads the 16-byte
// chunk 2*i + kg of its row.  A and B use the same assignment, so whichever k indices a
// lane's chunk holds, every k is multiplied with its partner exactly once.
//
// Accumulator layout of the 32x32 MFMAs: register r of lane l holds
//   C[row = 8*(r/4) + 4*(l>>5) + (r&3)][col = l & 31].
template <int DT>
struct Mma;

template <>
struct Mma<DT_BF16> {
  static __device__ __forceinline__ void run(f32x16& c, const uint4& a, const uint4& b) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};

template <>
struct Mma<DT_F32> {
  static __device__ __forceinline__ void run(f32x16& c, const uint4& a, const uint4& b) {
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
  }
};

__device__ __forceinline__ int acc_row(int r, int kg) { return 8 * (r >> 2) + 4 * kg + (r & 3); }

// m / n through the multiplier ceil(2^32 / n), exact while m * n < 2^32 (the multiplier exceeds 2^32 / n by
// less than 1, so the product exceeds m / n by less than m / 2^32 <= 1 / n); n == 1 has no 32-bit multiplier
// (it is passed as 0)
__device__ __forceinline__ int div_w(int m, uint32_t magic) { return magic ? (int)__umulhi((uint32_t)m, magic) : m; }

// Plane (within a 32-plane tile) that a hashing wave feeds as row rho of its A operand.  Accumulator
// register r of a lane in half kg is row 8*(r/4) + 4*kg + (r&3); with this order it is plane 16*kg + r,
// so a lane's 16 registers are 16 consecutive sign bits.
__device__ __forceinline__ int plane_row(int rho) { return 16 * ((rho >> 2) & 1) + 4 * (rho >> 3) + (rho & 3); }

// Workgroups are handed to the eight XCDs (each with its own L2) round-robin by linear id.  This maps
// id to an index whose consecutive values stay on one XCD: XCD x gets indices [x*n/8, (x+1)*n/8).
__device__ __forceinline__ int xcd_major(int id, int n) {
  return (n & 7) == 0 ? (id & 7) * (n >> 3) + (id >> 3) : id;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

__device__ __forceinline__ uint4 ld16(const void* p) { return *reinterpret_cast<const uint4*>(p); }

// 16-byte loads through a buffer descriptor: the address is a uniform base plus a 32-bit per-lane byte
// offset (no 64-bit address arithmetic per load), and offsets at or past `bytes` read as zero instead of
// touching memory, so rows beyond the end of a tensor need no clamping.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_srd(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
typedef uint32_t u32x4_ld __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 buf_ld16(__amdgpu_buffer_rsrc_t r, uint32_t byte_offset) {
  const u32x4_ld v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_offset, 0, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// Streaming stores: data that no later instruction of the same kernel reads goes out without waiting
// for the end-of-kernel write-back of the L2.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void st16_stream(void* p, const uint4& v) {
  u32x4 t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<u32x4*>(p));
}
template <typename T>
__device__ __forceinline__ void st_stream(T* p, T v) { __builtin_nontemporal_store(v, p); }

// inclusive prefix sum over the 64 lanes of a wave (DPP row shifts, then row broadcasts)
__device__ __forceinline__ int wave_incl_scan(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);  // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);  // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);  // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);  // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false); // row_bcast:15 into rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false); // row_bcast:31 into rows 2 and 3
  return v;
}

// Value of lane (l ^ 1), (l ^ 2), (l ^ 4) through DPP moves (no LDS round trip as a bpermute takes).
__device__ __forceinline__ uint32_t lane_xor1(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, true);  // quad_perm:[1,0,3,2]
}
__device__ __forceinline__ uint32_t lane_xor2(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, true);  // quad_perm:[2,3,0,1]
}
__device__ __forceinline__ uint32_t lane_xor4(uint32_t v, bool bit2) {
  const uint32_t up = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x104, 0xf, 0xf, true);    // row_shl:4: from lane l + 4
  const uint32_t down = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true);  // row_shr:4: from lane l - 4
  return bit2 ? down : up;
}
__device__ __forceinline__ float lane_xor1(float v) { return __uint_as_float(lane_xor1(__float_as_uint(v))); }
__device__ __forceinline__ float lane_xor2(float v) { return __uint_as_float(lane_xor2(__float_as_uint(v))); }
__device__ __forceinline__ int lane_xor1(int v) { return (int)lane_xor1((uint32_t)v); }
__device__ __forceinline__ int lane_xor2(int v) { return (int)lane_xor2((uint32_t)v); }
__device__ __forceinline__ int lane_xor4(int v, bool bit2) { return (int)lane_xor4((uint32_t)v, bit2); }
// Value of lane (l ^ 32): one swap of the wave's halves (upper: the lane is in the upper half), no LDS round trip.
__device__ __forceinline__ uint32_t half_other(uint32_t v, bool upper) {
  const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);  // r[0]: the lower half's values in all lanes, r[1]: the upper half's
  return upper ? r[0] : r[1];
}
__device__ __forceinline__ float half_other(float v, bool upper) { return __uint_as_float(half_other(__float_as_uint(v), upper)); }
// sum of a value over the lane pair (l, l ^ 32), the same bits in both lanes
__device__ __forceinline__ float half_pair_sum(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// max of a value over the lane pair (l, l ^ 32)
__device__ __forceinline__ float half_pair_max(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));  // r[0]: the lower half's values in all lanes, r[1]: the upper half's
}

// (m, s) pairs describe sum_i 2^(x_i) as s * 2^m.
__device__ __forceinline__ void lse_merge(float& m, float& s, float m2, float s2) {
  float mn = fmaxf(m, m2);
  s = s * fast_exp2(m - mn) + s2 * fast_exp2(m2 - mn);
  m = mn;
}

}  // namespace lkv
