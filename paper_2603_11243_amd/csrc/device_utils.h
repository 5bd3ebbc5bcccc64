// Small device helpers shared by the kernels: bf16 <-> fp32 bit moves, lane-group reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ssd {

typedef uint16_t bf16_t;   // raw bfloat16 bits

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round-to-nearest-even fp32 -> bf16 (finite inputs; NaN stays NaN)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// fp32 -> IEEE half bits, round to nearest even (v_cvt_f16_f32)
typedef uint16_t f16_t;    // raw IEEE binary16 bits
__device__ __forceinline__ f16_t f32_to_f16(float f) { return __builtin_bit_cast(f16_t, (_Float16)f); }
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
    return (uint32_t)f32_to_f16(lo) | ((uint32_t)f32_to_f16(hi) << 16);
}
__device__ __forceinline__ float f16_to_f32(f16_t v) { return (float)__builtin_bit_cast(_Float16, v); }

// Activation stores in half precision saturate: a value beyond the largest finite half (65504) is stored as
// +-65504 instead of +-inf, and `bad` remembers that it happened (also for NaN) so that the kernel can raise
// the sticky SSD_FLAG_ACT_OVERFLOW once at its end.  One compare and one v_med3_f32 per stored value.
constexpr float F16_MAX = 65504.0f;
__device__ __forceinline__ f16_t f32_to_f16_sat(float v, bool& bad) {
    bad |= !(fabsf(v) <= F16_MAX);
    return f32_to_f16(__builtin_amdgcn_fmed3f(v, -F16_MAX, F16_MAX));
}
__device__ __forceinline__ uint32_t pack_f16x2_sat(float lo, float hi, bool& bad) {
    return (uint32_t)f32_to_f16_sat(lo, bad) | ((uint32_t)f32_to_f16_sat(hi, bad) << 16);
}
// The same for kernels that store many values per lane: the common pass only tracks the largest magnitude
// (one v_max_f32 per value) and converts plainly; a lane that saw a value beyond the half range repeats
// its stores with f16_store<true>, which clamps.  (A NaN passes through both; it shows up as a non-finite
// likelihood, which raises the same flag.)
__device__ __forceinline__ float track_peak(float peak, float v) {
    float r;
    asm("v_max_f32 %0, %1, |%2|" : "=v"(r) : "v"(peak), "v"(v));
    return r;
}
template <bool CLAMP>
__device__ __forceinline__ f16_t f16_store(float v, float& peak) {
    if constexpr (CLAMP) return f32_to_f16(__builtin_amdgcn_fmed3f(v, -F16_MAX, F16_MAX));
    peak = track_peak(peak, v);
    return f32_to_f16(v);
}
template <bool CLAMP>
__device__ __forceinline__ uint32_t f16x2_store(float lo, float hi, float& peak) {
    return (uint32_t)f16_store<CLAMP>(lo, peak) | ((uint32_t)f16_store<CLAMP>(hi, peak) << 16);
}
// The 16-bit matrix-core operand type is a property of the context: IEEE half (BF = false: 11 significant bits,
// range 65504, stores saturate as above) or bfloat16 (BF = true: 8 significant bits, the range of fp32, nothing
// to saturate).  Kernels carry it as a template parameter; both are raw 16-bit patterns in memory.
template <bool BF> struct Op16;
template <> struct Op16<false> {
    static __device__ __forceinline__ uint16_t cvt(float v) { return f32_to_f16(v); }
    static __device__ __forceinline__ float to_f32(uint16_t b) { return f16_to_f32(b); }
    template <bool CLAMP> static __device__ __forceinline__ uint16_t store(float v, float& peak) { return f16_store<CLAMP>(v, peak); }
};
template <> struct Op16<true> {
    static __device__ __forceinline__ uint16_t cvt(float v) { return f32_to_bf16(v); }
    static __device__ __forceinline__ float to_f32(uint16_t b) { return bf16_to_f32(b); }
    template <bool CLAMP> static __device__ __forceinline__ uint16_t store(float v, float&) { return f32_to_bf16(v); }
};
template <bool BF> __device__ __forceinline__ uint32_t op_pack2(float lo, float hi) {
    return (uint32_t)Op16<BF>::cvt(lo) | ((uint32_t)Op16<BF>::cvt(hi) << 16);
}
template <bool BF, bool CLAMP> __device__ __forceinline__ uint32_t op_store2(float lo, float hi, float& peak) {
    return (uint32_t)Op16<BF>::template store<CLAMP>(lo, peak) | ((uint32_t)Op16<BF>::template store<CLAMP>(hi, peak) << 16);
}
// flag bits are those of enum ssd_device_flag (a vector atomic: several kernels may raise different bits)
__device__ __forceinline__ void raise_flag(int32_t* flags, int bit) {
    if (flags) atomicOr(flags, bit);
}

// Data-parallel-primitive lane moves inside a row of 16 lanes.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}
constexpr int DPP_XOR1 = 0xB1;          // quad_perm [1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;          // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141;  // lane i <-> 7-i inside each 8
constexpr int DPP_MIRROR = 0x140;       // lane i <-> 15-i inside each 16

struct OpMax { __device__ __forceinline__ float operator()(float a, float b) const { return fmaxf(a, b); } };
struct OpSum { __device__ __forceinline__ float operator()(float a, float b) const { return a + b; } };
struct OpMinI { __device__ __forceinline__ int operator()(int a, int b) const { return a < b ? a : b; } };

// All-reduce over groups of W consecutive lanes (W = 16 or 64); every lane gets the result.
template <int W, class Op>
__device__ __forceinline__ float group_allreduce(float v, Op op) {
    v = op(v, dpp_f<DPP_XOR1>(v));
    v = op(v, dpp_f<DPP_XOR2>(v));
    v = op(v, dpp_f<DPP_HALF_MIRROR>(v));
    v = op(v, dpp_f<DPP_MIRROR>(v));
    if (W > 16) {
        v = op(v, __shfl_xor(v, 16));
        v = op(v, __shfl_xor(v, 32));
    }
    return v;
}
template <int W, class Op>
__device__ __forceinline__ int group_allreduce_i(int v, Op op) {
    v = op(v, dpp_i<DPP_XOR1>(v));
    v = op(v, dpp_i<DPP_XOR2>(v));
    v = op(v, dpp_i<DPP_HALF_MIRROR>(v));
    v = op(v, dpp_i<DPP_MIRROR>(v));
    if (W > 16) {
        v = op(v, __shfl_xor(v, 16));
        v = op(v, __shfl_xor(v, 32));
    }
    return v;
}

// reduce over the 32 lanes of a half wavefront (same lane/32), e.g. the lanes that hold one row of
// a 32x32 MFMA accumulator block
template <class Op>
__device__ __forceinline__ float row_allreduce32(float v, Op op) {
    v = op(v, dpp_f<DPP_XOR1>(v));
    v = op(v, dpp_f<DPP_XOR2>(v));
    v = op(v, dpp_f<DPP_HALF_MIRROR>(v));
    v = op(v, dpp_f<DPP_MIRROR>(v));
    v = op(v, __shfl_xor(v, 16));
    return v;
}
__device__ __forceinline__ int row_allmin32_i(int v) {
    v = min(v, dpp_i<DPP_XOR1>(v));
    v = min(v, dpp_i<DPP_XOR2>(v));
    v = min(v, dpp_i<DPP_HALF_MIRROR>(v));
    v = min(v, dpp_i<DPP_MIRROR>(v));
    v = min(v, __shfl_xor(v, 16));
    return v;
}

}  // namespace ssd
