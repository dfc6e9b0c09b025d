// Shared device helpers for the gfx950 kernels: bf16 <-> float, 16-byte vector access,
// wave64 reductions.  Wavefronts are 64 lanes wide everywhere in this library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dicemoe {

constexpr int kWave = 64;
constexpr int kMaxExperts = 64;

typedef uint16_t bf16_t;  // raw bf16 bit pattern
// 16 bytes in four VGPRs.  Arrays of this native vector type stay in registers, whereas arrays of
// HIP's uint4 struct tend to be placed in scratch memory.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_to_float(bf16_t v) {
    return __uint_as_float(static_cast<uint32_t>(v) << 16);
}

// round-to-nearest-even; inputs are finite in every path that calls this
__device__ __forceinline__ bf16_t float_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<bf16_t>(u >> 16);
}

// two floats -> two bf16 in one register: the hardware conversion (v_cvt_pk_bf16_f32, round to
// nearest even, the same rounding as float_to_bf16 for finite values)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    const bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
    return *reinterpret_cast<const uint32_t*>(&r);
}

// storage-type traits: kVec elements fill 16 bytes
template <typename T> struct Store;
template <> struct Store<float> {
    static constexpr int kVec = 4;
    __device__ static __forceinline__ void unpack(const u32x4_t& v, float* f) {
        f[0] = __uint_as_float(v[0]); f[1] = __uint_as_float(v[1]);
        f[2] = __uint_as_float(v[2]); f[3] = __uint_as_float(v[3]);
    }
    __device__ static __forceinline__ void unpack(const uint4& v, float* f) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
        f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
    __device__ static __forceinline__ uint4 pack(const float* f) {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    }
};
template <> struct Store<bf16_t> {
    static constexpr int kVec = 8;
    __device__ static __forceinline__ void unpack(const u32x4_t& v, float* f) {
        f[0] = __uint_as_float(v[0] << 16); f[1] = __uint_as_float(v[0] & 0xFFFF0000u);
        f[2] = __uint_as_float(v[1] << 16); f[3] = __uint_as_float(v[1] & 0xFFFF0000u);
        f[4] = __uint_as_float(v[2] << 16); f[5] = __uint_as_float(v[2] & 0xFFFF0000u);
        f[6] = __uint_as_float(v[3] << 16); f[7] = __uint_as_float(v[3] & 0xFFFF0000u);
    }
    __device__ static __forceinline__ void unpack(const uint4& v, float* f) {
        f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
        f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
        f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xFFFF0000u);
        f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xFFFF0000u);
    }
    __device__ static __forceinline__ uint4 pack(const float* f) {
        return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]),
                          pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
    }
};

__device__ __forceinline__ int lane_id() { return static_cast<int>(threadIdx.x) & (kWave - 1); }

// butterfly sum over the 64 lanes: every lane ends with the same total, and the order of the
// additions is fixed, so results are reproducible run to run
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, kWave));
    return v;
}

__device__ __forceinline__ uint64_t lanemask_lt() {
    return (1ull << lane_id()) - 1ull;
}

}  // namespace dicemoe
