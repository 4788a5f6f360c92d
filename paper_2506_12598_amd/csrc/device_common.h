// Device-side helpers shared by the kernels of libeclip (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace eclip {

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>).  Unlike `#pragma unroll`
// it cannot be declined by the unroller's size threshold, which matters where a loop index selects an
// accumulator register: a loop left rolled there sends the whole accumulator array to scratch memory.
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F &f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

enum { ACT_NONE = 0, ACT_RELU = 1, ACT_RELU6 = 2, ACT_GELU = 3 };

// 16-bit storage types are carried as raw bit patterns; the tag types select the conversions.
struct bf16_t { uint16_t bits; };
struct f16_t { uint16_t bits; };

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
// float -> bfloat16, round to nearest even: gfx950 has the conversion in hardware (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f);
}
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
// two floats -> two 16-bit values in one word (a in the low half)
__device__ __forceinline__ uint32_t f32x2_to_bf16x2_bits(float a, float b)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){a, b}, bf16x2));
}
__device__ __forceinline__ uint32_t f32x2_to_f16x2_bits(float a, float b)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){a, b}, f16x2));
}
__device__ __forceinline__ float f16_bits_to_f32(uint32_t b)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)b);
}
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f)
{
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
}

template <typename T> struct Cvt;
template <> struct Cvt<float> {
    static constexpr int VEC = 4;                                 // elements per 16-byte access
    __device__ static __forceinline__ float load(const float *p) { return *p; }
    __device__ static __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Cvt<bf16_t> {
    static constexpr int VEC = 8;
    __device__ static __forceinline__ float load(const bf16_t *p) { return bf16_bits_to_f32(p->bits); }
    __device__ static __forceinline__ void store(bf16_t *p, float v) { p->bits = (uint16_t)f32_to_bf16_bits(v); }
    __device__ static __forceinline__ float from_bits(uint32_t b) { return bf16_bits_to_f32(b); }
    __device__ static __forceinline__ uint32_t to_bits(float v) { return f32_to_bf16_bits(v); }
    __device__ static __forceinline__ uint32_t pack2(float a, float b) { return f32x2_to_bf16x2_bits(a, b); }
};
template <> struct Cvt<f16_t> {
    static constexpr int VEC = 8;
    __device__ static __forceinline__ float load(const f16_t *p) { return f16_bits_to_f32(p->bits); }
    __device__ static __forceinline__ void store(f16_t *p, float v) { p->bits = (uint16_t)f32_to_f16_bits(v); }
    __device__ static __forceinline__ float from_bits(uint32_t b) { return f16_bits_to_f32(b); }
    __device__ static __forceinline__ uint32_t to_bits(float v) { return f32_to_f16_bits(v); }
    __device__ static __forceinline__ uint32_t pack2(float a, float b) { return f32x2_to_f16x2_bits(a, b); }
};

// V consecutive elements <-> V floats.  V == Cvt<T>::VEC uses one 16-byte access, V == 4 of a 16-bit type an 8-byte
// one, V == 1 a scalar one.
template <typename T, int V> struct Pack {
    __device__ static __forceinline__ void load(const T *p, float (&v)[V])
    {
        if constexpr (V == 1) {
            v[0] = Cvt<T>::load(p);
        } else if constexpr (sizeof(T) == 4) {
            const float4 q = *reinterpret_cast<const float4 *>(p);
            v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
        } else if constexpr (V == 4) {               // four 16-bit elements: one 8-byte access
            const uint2 q = *reinterpret_cast<const uint2 *>(p);
            v[0] = Cvt<T>::from_bits(q.x & 0xffffu); v[1] = Cvt<T>::from_bits(q.x >> 16);
            v[2] = Cvt<T>::from_bits(q.y & 0xffffu); v[3] = Cvt<T>::from_bits(q.y >> 16);
        } else {
            const uint4 q = *reinterpret_cast<const uint4 *>(p);
            const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[2 * i] = Cvt<T>::from_bits(w[i] & 0xffffu);
                v[2 * i + 1] = Cvt<T>::from_bits(w[i] >> 16);
            }
        }
    }
    __device__ static __forceinline__ void store(T *p, const float (&v)[V])
    {
        if constexpr (V == 1) {
            Cvt<T>::store(p, v[0]);
        } else if constexpr (sizeof(T) == 4) {
            *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
        } else if constexpr (V == 4) {
            *reinterpret_cast<uint2 *>(p) = make_uint2(Cvt<T>::pack2(v[0], v[1]), Cvt<T>::pack2(v[2], v[3]));
        } else {
            uint32_t w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) w[i] = Cvt<T>::pack2(v[2 * i], v[2 * i + 1]);
            *reinterpret_cast<uint4 *>(p) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
};

// GELU with the exact-erf definition, v Phi(v) = v / 2 (1 + erf(v / sqrt 2)), to about 3e-7 absolute.  erf comes from
// the rational form 1 - (a1 t + ... + a5 t^5) exp(-x^2), t = 1 / (1 + p |x|) (Abramowitz & Stegun 7.1.26, error below
// 1.5e-7 in exact arithmetic), with the hardware reciprocal and exp2.  Written out for x = |v| / sqrt 2 the two signs
// give one expression,
//     v Phi(v) = max(v, 0) - |v| (a1 t + ... + a5 t^5) / 2 * exp(-v^2 / 2),
// which needs no sign transfer, keeps its relative accuracy in the negative tail (no 1 - erf cancellation) and takes 13
// instructions, two of them quarter-rate; the library erff takes about three times as many, which made an element-wise
// GELU ALU-bound, and in a GEMM epilogue nothing else runs on the CU while the vector ALU works through the tile.
__device__ __forceinline__ float gelu_erf(float v)
{
    const float av = fabsf(v);
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752440f, av, 1.0f));
    float q = fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
    q = fmaf(q, t, 0.5f * 1.421413741f);
    q = fmaf(q, t, 0.5f * -0.284496736f);
    q = fmaf(q, t, 0.5f * 0.254829592f);
    const float e = __builtin_amdgcn_exp2f((-0.5f * 1.4426950408889634f * v) * v);
    return fmaf(-(q * t * e), av, fmaxf(v, 0.0f));
}

__device__ __forceinline__ float apply_act(int act, float v)
{
    switch (act) {
    case ACT_RELU:  return fmaxf(v, 0.0f);
    case ACT_RELU6: return fminf(fmaxf(v, 0.0f), 6.0f);
    case ACT_GELU:  return gelu_erf(v);
    default:        return v;
    }
}

// The same with the activation fixed at compile time.  A kernel's epilogue is unrolled over its accumulator blocks, and
// with a run-time switch every copy carries the code of all activations: the code that runs then hops over the code
// that does not, which defeats the sequential instruction prefetch (measured: a 256 x 256 tile kernel of 146 KB, 52 KB
// without the switches, lost 5.6 us per launch to instruction-cache misses at its start).  Kernels therefore branch on
// the activation once, with ECLIP_ACT_SWITCH, into epilogues that each hold one activation.
template <int ACT>
__device__ __forceinline__ float apply_act_c(float v)
{
    if constexpr (ACT == ACT_RELU) return fmaxf(v, 0.0f);
    else if constexpr (ACT == ACT_RELU6) return fminf(fmaxf(v, 0.0f), 6.0f);
    else if constexpr (ACT == ACT_GELU) return gelu_erf(v);
    else return v;
}
#define ECLIP_ACT_SWITCH(act, CALL)          \
    switch (act) {                           \
    case ACT_RELU:  CALL(ACT_RELU); break;   \
    case ACT_RELU6: CALL(ACT_RELU6); break;  \
    case ACT_GELU:  CALL(ACT_GELU); break;   \
    default:        CALL(ACT_NONE); break;   \
    }

// Sum / max over the 64 lanes of a wavefront; every lane receives the result.
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// The same over aligned groups of W lanes (W = 16, 32 or 64): every lane receives the result of its own group.
template <int W>
__device__ __forceinline__ float group_sum(float v)
{
#pragma unroll
    for (int o = W / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
template <int W>
__device__ __forceinline__ float group_max(float v)
{
#pragma unroll
    for (int o = W / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

}  // namespace eclip
