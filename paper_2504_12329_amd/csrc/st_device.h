// Device-side helpers shared by the HIP kernels of the library (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace st {

constexpr int kWave = 64;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // one 16-byte global load

// Slots of the per-model device state block (int32 each).
enum StateSlot {
    kPos = 0,    // position the next fed token will take (== number of cached positions)
    kTok = 1,    // last greedy token
    kFired = 2,  // 1 if the trigger rule fired on kTok
    kFed = 3,    // token fed by the step that produced kTok
    kStep = 4,   // running index into the output-token buffer of a chained run
    kCount = 5,  // scratch counter of set-up kernels (weights an fp16 copy could not hold)
    kEpoch = 6,  // launches of the persistent decode step so far (its hand-over words carry epochs derived from it)
    kPersistErr = 7,  // 1 once a wait inside the persistent decode step has timed out
    kStateInts = 16
};

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// fp32 -> bf16, round to nearest even, NaN stays NaN: the hardware conversion (v_cvt_pk_bf16_f32).
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Cross-lane reductions without the LDS crossbar (a ds_bpermute step costs ~60 clocks of latency, a DPP step ~8):
// quad swaps, half-row and row mirrors, then the two row broadcasts leave the total in lane 63, which is read back
// to every lane.  `old` is what a lane keeps where the pattern has no source for it (the reduction's identity).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float old, float v) {
    return __int_as_float(
        __builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_move<0xB1, 0xf>(0.f, v);   // quad_perm [1,0,3,2]
    v += dpp_move<0x4E, 0xf>(0.f, v);   // quad_perm [2,3,0,1]
    v += dpp_move<0x141, 0xf>(0.f, v);  // row_half_mirror
    v += dpp_move<0x140, 0xf>(0.f, v);  // row_mirror: every lane holds its row's sum
    v += dpp_move<0x142, 0xa>(0.f, v);  // row_bcast15 into rows 1 and 3
    v += dpp_move<0x143, 0xc>(0.f, v);  // row_bcast31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_move<0xB1, 0xf>(-INFINITY, v));
    v = fmaxf(v, dpp_move<0x4E, 0xf>(-INFINITY, v));
    v = fmaxf(v, dpp_move<0x141, 0xf>(-INFINITY, v));
    v = fmaxf(v, dpp_move<0x140, 0xf>(-INFINITY, v));
    v = fmaxf(v, dpp_move<0x142, 0xa>(-INFINITY, v));
    v = fmaxf(v, dpp_move<0x143, 0xc>(-INFINITY, v));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
// x[lane] and x[lane ^ 16] / x[lane ^ 32], by swapping 16- / 32-lane rows of two copies of the register
typedef unsigned int lane_pair_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void with_xor16(float x, float &a, float &b) {
    const lane_pair_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    a = __uint_as_float(r.x), b = __uint_as_float(r.y);
}
__device__ __forceinline__ void with_xor32(float x, float &a, float &b) {
    const lane_pair_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    a = __uint_as_float(r.x), b = __uint_as_float(r.y);
}
__device__ __forceinline__ float sum_xor16(float x) {
    float a, b;
    with_xor16(x, a, b);
    return a + b;
}
__device__ __forceinline__ float sum_xor32(float x) {
    float a, b;
    with_xor32(x, a, b);
    return a + b;
}
__device__ __forceinline__ float max_xor32(float x) {
    float a, b;
    with_xor32(x, a, b);
    return fmaxf(a, b);
}

// Sum over a 256-thread block (4 waves); `red` is 4 floats of LDS.  Ends with a barrier.
__device__ __forceinline__ float block_sum_256(float v, float *red) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

// fma of 8 bf16 weights (one 16-byte load) with 8 fp32 activations.
__device__ __forceinline__ float dot8(const u32x4 &w, const float4 &xa, const float4 &xb, float acc) {
    acc = fmaf(bf16_lo(w.x), xa.x, acc);
    acc = fmaf(bf16_hi(w.x), xa.y, acc);
    acc = fmaf(bf16_lo(w.y), xa.z, acc);
    acc = fmaf(bf16_hi(w.y), xa.w, acc);
    acc = fmaf(bf16_lo(w.z), xb.x, acc);
    acc = fmaf(bf16_hi(w.z), xb.y, acc);
    acc = fmaf(bf16_lo(w.w), xb.z, acc);
    acc = fmaf(bf16_hi(w.w), xb.w, acc);
    return acc;
}

}  // namespace st
