// Device-side helpers shared by the gfx950 kernels: storage-type conversion,
// wavefront (64-lane) and workgroup reductions, Philox4x32-10.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace xsm {

// bf16 storage element (bit pattern); arithmetic is always fp32.
struct bf16_t { uint16_t x; };

__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// round-to-nearest-even, on gfx950's conversion instruction (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint16_t f2bf(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
// (a, b) -> bf16 pair, a in the low half
__device__ __forceinline__ uint32_t f2bf_pair(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{a, b}, bf16x2_t));
}
// four floats -> packed bf16 pairs of the rounded values (hi) and of what the rounding dropped (lo)
__device__ __forceinline__ void split4(const float4 v, uint2& hi, uint2& lo) {
  hi = uint2{f2bf_pair(v.x, v.y), f2bf_pair(v.z, v.w)};
  lo = uint2{f2bf_pair(v.x - __uint_as_float(hi.x << 16), v.y - __uint_as_float(hi.x & 0xFFFF0000u)),
             f2bf_pair(v.z - __uint_as_float(hi.y << 16), v.w - __uint_as_float(hi.y & 0xFFFF0000u))};
}

// Activation rows as MFMA operands: bf16 hi and lo planes in fragment order.  A tile of 16 rows x
// 32 contraction indices is one contiguous KB in which lane (row & 15) + 16 * ((k >> 3) & 3) holds 8
// consecutive k, tiles ordered [row tile][k tile]: a wavefront fetches a whole "B" fragment as one
// contiguous KB.  (With row-major planes a fragment is 16 rows x 64 B, and the GEMMs that read
// them straight from L2 took 30 % longer.)  A plane covers whole 16-row tiles; rows past M are
// never written and feed only MFMA columns that are never stored.
__host__ __device__ __forceinline__ size_t plane_elems(int M, int K) { return (size_t)((M + 15) & ~15) * K; }
__device__ __forceinline__ size_t plane_index(int K, int m, int k) {
  return ((size_t)((m >> 4) * (K >> 5) + (k >> 5)) * 64 + (m & 15) + 16 * ((k >> 3) & 3)) * 8 + (k & 7);
}
// v = columns k..k+3 (k % 4 == 0) of row m of an [M][K] activation block -> both planes at `planes`
__device__ __forceinline__ void plane_store4(void* planes, int M, int K, int m, int k, float4 v) {
  uint2 hi, lo;
  split4(v, hi, lo);
  uint16_t* hp = reinterpret_cast<uint16_t*>(planes) + plane_index(K, m, k);
  *reinterpret_cast<uint2*>(hp) = hi;
  *reinterpret_cast<uint2*>(hp + plane_elems(M, K)) = lo;
}
__device__ __forceinline__ float ldf(const float* p) { return *p; }
__device__ __forceinline__ float ldf(const bf16_t* p) { return bf2f(p->x); }
__device__ __forceinline__ void stf(float* p, float v) { *p = v; }
__device__ __forceinline__ void stf(bf16_t* p, float v) { p->x = f2bf(v); }

// Load VEC consecutive storage elements (16-byte aligned) as floats.
__device__ __forceinline__ void ldvec(const float* p, float (&o)[4]) {
  float4 v = *reinterpret_cast<const float4*>(p);
  o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
}
__device__ __forceinline__ void ldvec(const bf16_t* p, float (&o)[8]) {
  uint4 v = *reinterpret_cast<const uint4*>(p);
  o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xFFFF0000u);
  o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xFFFF0000u);
  o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xFFFF0000u);
  o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xFFFF0000u);
}
template <typename T> struct VecOf;
template <> struct VecOf<float> { static constexpr int n = 4; };
template <> struct VecOf<bf16_t> { static constexpr int n = 8; };

constexpr int WAVE = 64;

// Value held by lane (l ^ MASK), MASK a power of two, without the LDS crossbar that __shfl_xor
// goes through (ds_bpermute: an address computation plus LDS latency per exchange): the lane-swap
// instructions of gfx950 for 32 and 16, DPP row operations for 8 and below.  All 64 lanes must
// be active and blockDim.x a multiple of 64.  (Lane layouts checked on gfx950 against __shfl_xor.)
template <int MASK>
__device__ __forceinline__ uint32_t lane_xor_u32(uint32_t x) {
  static_assert(MASK == 1 || MASK == 2 || MASK == 4 || MASK == 8 || MASK == 16 || MASK == 32, "one lane bit");
  if constexpr (MASK == 32) {
    const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return (threadIdx.x & 32) ? r[0] : r[1];
  } else if constexpr (MASK == 16) {
    const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    return (threadIdx.x & 16) ? r[0] : r[1];
  } else if constexpr (MASK == 8) {
    return __builtin_amdgcn_update_dpp(0u, x, 0x128, 0xf, 0xf, false);          // row_ror:8
  } else if constexpr (MASK == 4) {
    const uint32_t y = __builtin_amdgcn_update_dpp(0u, x, 0x141, 0xf, 0xf, false);   // row_half_mirror: lane 7 - i of the eight
    return __builtin_amdgcn_update_dpp(0u, y, 0x1B, 0xf, 0xf, false);           // quad_perm [3,2,1,0]
  } else if constexpr (MASK == 2) {
    return __builtin_amdgcn_update_dpp(0u, x, 0x4E, 0xf, 0xf, false);           // quad_perm [2,3,0,1]
  } else {
    return __builtin_amdgcn_update_dpp(0u, x, 0xB1, 0xf, 0xf, false);           // quad_perm [1,0,3,2]
  }
}
template <int MASK> __device__ __forceinline__ float lane_xor(float x) {
  return __uint_as_float(lane_xor_u32<MASK>(__float_as_uint(x)));
}
template <int MASK> __device__ __forceinline__ int lane_xor(int x) { return (int)lane_xor_u32<MASK>((uint32_t)x); }

// every lane receives the result; fixed combination order (lane distance 32, 16, ..., 1)
__device__ __forceinline__ float wave_sum(float v) {
  v += lane_xor<32>(v); v += lane_xor<16>(v); v += lane_xor<8>(v);
  v += lane_xor<4>(v); v += lane_xor<2>(v); v += lane_xor<1>(v);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, lane_xor<32>(v)); v = fmaxf(v, lane_xor<16>(v)); v = fmaxf(v, lane_xor<8>(v));
  v = fmaxf(v, lane_xor<4>(v)); v = fmaxf(v, lane_xor<2>(v)); v = fmaxf(v, lane_xor<1>(v));
  return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
  v += lane_xor<32>(v); v += lane_xor<16>(v); v += lane_xor<8>(v);
  v += lane_xor<4>(v); v += lane_xor<2>(v); v += lane_xor<1>(v);
  return v;
}
__device__ __forceinline__ int wave_min_i(int v) {
  v = min(v, lane_xor<32>(v)); v = min(v, lane_xor<16>(v)); v = min(v, lane_xor<8>(v));
  v = min(v, lane_xor<4>(v)); v = min(v, lane_xor<2>(v)); v = min(v, lane_xor<1>(v));
  return v;
}
__device__ __forceinline__ int wave_max_i(int v) {
  v = max(v, lane_xor<32>(v)); v = max(v, lane_xor<16>(v)); v = max(v, lane_xor<8>(v));
  v = max(v, lane_xor<4>(v)); v = max(v, lane_xor<2>(v)); v = max(v, lane_xor<1>(v));
  return v;
}

// Workgroup reductions for blockDim.x == 256 (4 wavefronts); red points to >= 8
// floats of LDS.  All threads receive the result.  Fixed combination order.
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}
__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}
__device__ __forceinline__ int block_sum_i(int v, int* red) {
  v = wave_sum_i(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}
__device__ __forceinline__ int block_min_i(int v, int* red) {
  v = wave_min_i(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return min(min(red[0], red[1]), min(red[2], red[3]));
}
__device__ __forceinline__ int block_max_i(int v, int* red) {
  v = wave_max_i(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return max(max(red[0], red[1]), max(red[2], red[3]));
}

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies,
// key words bumped by Weyl constants between rounds.
__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint2 k) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { k.x += 0x9E3779B9u; k.y += 0xBB67AE85u; }
    const uint32_t hi0 = __umulhi(0xD2511F53u, c.x), lo0 = 0xD2511F53u * c.x;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c.z), lo1 = 0xCD9E8D57u * c.z;
    c = make_uint4(hi1 ^ c.y ^ k.x, lo1, hi0 ^ c.w ^ k.y, lo0);
  }
  return c;
}
// Uniform in [0,1) with 24 bits; counter (position, head, sequence id, 0).
__device__ __forceinline__ float philox_uniform(uint64_t seed, uint32_t pos, uint32_t head,
                                                uint32_t seq) {
  const uint4 o = philox4x32_10(make_uint4(pos, head, seq, 0u),
                                make_uint2((uint32_t)seed, (uint32_t)(seed >> 32)));
  return (float)(o.x >> 8) * (1.0f / 16777216.0f);
}

}  // namespace xsm
