// Pieces shared by the two matrix-core GEMM kernels: the argument block, the MFMA wrappers and the
// bias / residual / activation epilogue.
#pragma once
#include "device_common.h"

namespace eclip {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct GemmDev {
    const uint16_t *x, *w, *bias, *res;
    uint16_t *y;
    float *y32;
    float *ws;
    int B, H, W, Cin, Ho, Wo, KH, KW, stride, pad, act;
    int M, N, K, KT, kt_per, splits, tiles_m, tiles_n, raster;
    unsigned x_bytes, w_bytes;               // sizes of the x and w tensors (each below 4 GiB)
    int nchw_c;                              // > 0: x is the caller's [B][nchw_c][H][W] tensor (first layer), Cin == 8
    int ldx, ldy;                            // elements between consecutive pixels of x / rows of y (Cin and N unless the tensor is
                                             // a channel range of a wider buffer: concatenation in place); res is null when ldy != N
};

template <typename T> struct Mma;
template <> struct Mma<bf16_t> {
    __device__ static __forceinline__ f32x4 run(uint4 a, uint4 b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mma<f16_t> {
    __device__ static __forceinline__ f32x4 run(uint4 a, uint4 b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};

// bias + residual + activation + store of 4 consecutive channels n..n+3 of output row m
template <typename T, int ACT>
__device__ __forceinline__ void epilogue_store(const uint16_t *bias, const uint16_t *res, uint16_t *y, float *y32,
                                               int M, int N, int m, int n, f32x4 v, int nvalid = 4, int ld = 0)
{
    if (m >= M || n >= N) return;
    const long off = (long)m * (ld ? ld : N) + n;      // ld: row pitch of y when it differs from N (a multiple of 8)
    float o[4] = {v[0], v[1], v[2], v[3]};
    if ((N & 3) == 0 && nvalid == 4) {       // then n + 3 < N and every access below is aligned
        if (bias) {
            const uint2 q = *reinterpret_cast<const uint2 *>(bias + n);
            o[0] += Cvt<T>::from_bits(q.x & 0xffffu); o[1] += Cvt<T>::from_bits(q.x >> 16);
            o[2] += Cvt<T>::from_bits(q.y & 0xffffu); o[3] += Cvt<T>::from_bits(q.y >> 16);
        }
        if (res) {
            const uint2 q = *reinterpret_cast<const uint2 *>(res + off);
            o[0] += Cvt<T>::from_bits(q.x & 0xffffu); o[1] += Cvt<T>::from_bits(q.x >> 16);
            o[2] += Cvt<T>::from_bits(q.y & 0xffffu); o[3] += Cvt<T>::from_bits(q.y >> 16);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) o[r] = apply_act_c<ACT>(o[r]);
        if (y32) {
            *reinterpret_cast<float4 *>(y32 + off) = make_float4(o[0], o[1], o[2], o[3]);
        } else {
            uint2 q;
            q.x = Cvt<T>::pack2(o[0], o[1]);
            q.y = Cvt<T>::pack2(o[2], o[3]);
            *reinterpret_cast<uint2 *>(y + off) = q;
        }
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (r >= nvalid || n + r >= N) break;
            float t = o[r];
            if (bias) t += Cvt<T>::from_bits(bias[n + r]);
            if (res) t += Cvt<T>::from_bits(res[off + r]);
            t = apply_act_c<ACT>(t);
            if (y32) y32[off + r] = t;
            else y[off + r] = (uint16_t)Cvt<T>::to_bits(t);
        }
    }
}

// The same for 8 consecutive channels n..n+7 of row m, with 16-byte accesses: requires N % 8 == 0, n % 8 == 0,
// m < M and n < N (checked by the caller).  `o` holds the sums without bias; ld = row pitch of y (and of res).
template <typename T, int ACT>
__device__ __forceinline__ void epilogue_store8(const uint16_t *bias, const uint16_t *res, uint16_t *y, float *y32, int ld,
                                                int m, int n, float (&o)[8])
{
    const long off = (long)m * ld + n;
    if (bias) {
        float bv[8];
        Pack<T, 8>::load(reinterpret_cast<const T *>(bias) + n, bv);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] += bv[e];
    }
    if (res) {
        float rv[8];
        Pack<T, 8>::load(reinterpret_cast<const T *>(res) + off, rv);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] += rv[e];
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = apply_act_c<ACT>(o[e]);
    if (y32) {
        *reinterpret_cast<float4 *>(y32 + off) = make_float4(o[0], o[1], o[2], o[3]);
        *reinterpret_cast<float4 *>(y32 + off + 4) = make_float4(o[4], o[5], o[6], o[7]);
    } else {
        Pack<T, 8>::store(reinterpret_cast<T *>(y) + off, o);
    }
}

// The same for any N: channels n..n+7 of row m that lie below N, one element at a time.
template <typename T, int ACT>
__device__ __forceinline__ void epilogue_store8_ragged(const uint16_t *bias, const uint16_t *res, uint16_t *y, float *y32, int N, int ld,
                                                       int m, int n, const float (&o)[8])
{
    const long off = (long)m * ld + n;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (n + e >= N) break;
        float t = o[e];
        if (bias) t += Cvt<T>::from_bits(bias[n + e]);
        if (res) t += Cvt<T>::from_bits(res[off + e]);
        t = apply_act_c<ACT>(t);
        if (y32) y32[off + e] = t;
        else y[off + e] = (uint16_t)Cvt<T>::to_bits(t);
    }
}

// wave-split-K kernel (k_wsk.hip)
hipError_t launch_conv_wsk(const GemmDev &d, int dtype, int variant, int nw, int tiles, hipStream_t s);
// two independent layers of the same tile shape and wavefront count in one launch
hipError_t launch_conv_wsk_pair(const GemmDev &d0, int tiles0, const GemmDev &d1, int tiles1, int dtype, int variant, int nw, hipStream_t s);

}  // namespace eclip
