// Small device-side helpers shared by the gfx950 kernels: element types, 16-byte typed
// loads widened to fp32, wavefront (64-lane) and lane-group reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace shk {

typedef _Float16 f16_t;   // IEEE half: the 16-bit format of activations and of the KV cache

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int VEC = 4;  // elements per 16-byte load
    __device__ static __forceinline__ float to_f32(float v) { return v; }
    __device__ static __forceinline__ float from_f32(float v) { return v; }
};
template <> struct Elem<f16_t> {
    static constexpr int VEC = 8;
    __device__ static __forceinline__ float to_f32(f16_t v) { return static_cast<float>(v); }
    __device__ static __forceinline__ f16_t from_f32(float v) { return static_cast<f16_t>(v); }
};

// Rounding an activation or cache value to its stored type.  IEEE half ends at 65504: a value
// beyond it (or a NaN) sets *oflow, a word in host-visible memory that the runtime tests
// before every call (plain store of the same value from every lane that sees one: no atomic
// needed, and no traffic at all in the normal case).  fp32 stores pass through.
template <typename T>
__device__ __forceinline__ T store_cast(float v, uint32_t* oflow);
template <>
__device__ __forceinline__ float store_cast<float>(float v, uint32_t*) { return v; }
template <>
__device__ __forceinline__ f16_t store_cast<f16_t>(float v, uint32_t* oflow) {
    if (!(fabsf(v) <= 65504.0f)) *oflow = 1u;
    return static_cast<f16_t>(v);
}

// Activation / KV-cache element type that goes with a weight element type.
template <typename WT> struct ActOf;
template <> struct ActOf<float> { typedef float type; };
template <> struct ActOf<f16_t> { typedef f16_t type; };

// Load 16 bytes at p (16-byte aligned) and widen to fp32: 4 floats or 8 halfs.
template <typename T> struct Vec16;
// load_stream: the same with a non-temporal hint, for data read exactly once (weights of the
// autoregressive phase) - measured 4-6 % faster streams than plain loads on MI355X.
template <> struct Vec16<float> {
    float v[4];
    __device__ __forceinline__ void load(const float* p) {
        const float4 t = *reinterpret_cast<const float4*>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
    __device__ __forceinline__ void load_stream(const float* p) {
        const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
        v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
    }
    __device__ __forceinline__ void zero() { v[0] = v[1] = v[2] = v[3] = 0.f; }
};
template <> struct Vec16<f16_t> {
    float v[8];
    __device__ __forceinline__ void load(const f16_t* p) {
        typedef _Float16 h8 __attribute__((ext_vector_type(8)));
        const h8 t = *reinterpret_cast<const h8*>(p);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = static_cast<float>(t[i]);
    }
    __device__ __forceinline__ void load_stream(const f16_t* p) {
        typedef _Float16 h8 __attribute__((ext_vector_type(8)));
        const h8 t = __builtin_nontemporal_load(reinterpret_cast<const h8*>(p));
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = static_cast<float>(t[i]);
    }
    __device__ __forceinline__ void zero() {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = 0.f;
    }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Sequences of one call, passed by value in the kernel arguments.
// Sum over groups of TPT adjacent lanes (TPT a power of two; groups aligned to TPT), the
// result in every lane of the group.  Within a row of 16 lanes the exchanges are DPP
// modifiers of the add itself (quad permutes, then the half-row and row mirrors), which cost
// no LDS-crossbar instruction; only steps across rows use a shuffle.
template <int CTRL>
__device__ __forceinline__ float dpp_read(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
template <int TPT>
__device__ __forceinline__ float group_sum(float v) {
    if constexpr (TPT >= 2) v += dpp_read<0xB1>(v);    // quad_perm [1,0,3,2]
    if constexpr (TPT >= 4) v += dpp_read<0x4E>(v);    // quad_perm [2,3,0,1]
    if constexpr (TPT >= 8) v += dpp_read<0x141>(v);   // row_half_mirror
    if constexpr (TPT >= 16) v += dpp_read<0x140>(v);  // row_mirror
    if constexpr (TPT >= 32) v += __shfl_xor(v, 16, 64);
    if constexpr (TPT >= 64) v += __shfl_xor(v, 32, 64);
    return v;
}

// Sum over the 64 lanes of a wave, the result in every lane, without the LDS crossbar: rows of 16
// lanes by DPP (group_sum<16>), then the four row sums through scalar registers.  Used at the end
// of the streaming projections, where a chain of six dependent cross-lane shuffles per value
// was a visible part of every launch.
__device__ __forceinline__ float wave_sum_rows(float v) {
    v = group_sum<16>(v);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
    return (r0 + r1) + (r2 + r3);
}

// Direct global -> LDS load (global_load_lds_dwordx4, gfx950): lds_byte (wave-uniform) goes to M0
// and lane l's 16 bytes land at lds_byte + 16 * l; no registers are occupied while the load is
// in flight.  Inline assembly because the compiler, for its own direct-to-LDS builtin, waits for
// every outstanding load before any LDS read; users wait explicitly with wait_vmcnt.
__device__ __forceinline__ void lds_dma16(const void* g, uint32_t lds_byte) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_byte) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// pos[b] = tokens already cached for seq[b] before this call.
struct SeqBatch {
    int32_t n;
    int32_t seq[64];
    int32_t pos[64];
};

}  // namespace shk
