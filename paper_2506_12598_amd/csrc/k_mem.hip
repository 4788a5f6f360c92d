// Memory-bound kernels: float32 direct convolution, depthwise convolution, pooling, LayerNorm,
// softmax, element-wise epilogue, embedding gather and the layout conversions at the model boundary.
// All activations are channels-last; every thread moves 16 bytes per access when the channel count
// allows it (V = 8 sixteen-bit or 4 float elements), else one element (V = 1).
#include "device_common.h"
#include "kernels.h"

namespace eclip {

namespace {

// Workgroup b runs on XCD b % 8, and each XCD has an L2 of its own.  A sliding-window kernel whose neighbouring
// workgroups read overlapping input rows therefore numbers its work in 8 contiguous bands, one per XCD, so that the
// overlap is fetched from HBM once and found in that XCD's L2 afterwards (measured on a 3x3 depth-wise convolution of
// 192 x 1120 x 1120: HBM reads of 3.1x the input with round-robin numbering).  gridDim.x must be a multiple of 8.
__device__ __forceinline__ unsigned banded_block() { return (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3); }

inline unsigned blocks_for(long n_threads, int block) { return (unsigned)((n_threads + block - 1) / block); }
// grid for a kernel that numbers its workgroups with banded_block(): a multiple of 8
inline unsigned banded_blocks_for(long n_threads, int block) { return (blocks_for(n_threads, block) + 7u) & ~7u; }

// Dispatch on dtype and on whether `width` allows 16-byte accesses.
#define ECLIP_DISPATCH(dtype, width, CALL)                                         \
    do {                                                                           \
        if ((dtype) == DT_F32) {                                                   \
            if ((width) % 4 == 0) { CALL(float, 4); } else { CALL(float, 1); }     \
        } else if ((dtype) == DT_BF16) {                                           \
            if ((width) % 8 == 0) { CALL(bf16_t, 8); } else { CALL(bf16_t, 1); }   \
        } else {                                                                   \
            if ((width) % 8 == 0) { CALL(f16_t, 8); } else { CALL(f16_t, 1); }     \
        }                                                                          \
    } while (0)

// ---------------- float32 direct convolution: one thread per output element ----------------------
__global__ __launch_bounds__(256) void conv_f32_kernel(ConvF32Args a, long total)
{
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const unsigned ui = (unsigned)idx;
    const int n = (int)(ui % (unsigned)a.Cout);
    const unsigned m = ui / (unsigned)a.Cout;
    const int ow = (int)(m % (unsigned)a.Wo);
    const unsigned mh = m / (unsigned)a.Wo;
    const int oh = (int)(mh % (unsigned)a.Ho);
    const int b = (int)(mh / (unsigned)a.Ho);
    float acc = a.bias ? a.bias[n] : 0.0f;
    for (int kh = 0; kh < a.KH; ++kh) {
        const int ih = oh * a.stride - a.pad + kh;
        if ((unsigned)ih >= (unsigned)a.H) continue;
        for (int kw = 0; kw < a.KW; ++kw) {
            const int iw = ow * a.stride - a.pad + kw;
            if ((unsigned)iw >= (unsigned)a.W) continue;
            const float *xp = a.x + (((long)b * a.H + ih) * a.W + iw) * a.Cin;
            const float *wp = a.w + ((long)(kh * a.KW + kw) * a.Cin) * a.Cout + n;
            for (int ci = 0; ci < a.Cin; ++ci) acc = fmaf(xp[ci], wp[(long)ci * a.Cout], acc);
        }
    }
    if (a.res) acc += a.res[idx];
    a.y[idx] = apply_act(a.act, acc);
}

// ---------------- depthwise convolution --------------------------------------------------------------
// One thread per (output pixel, V channels).  KS > 0 fixes the window size at compile time so that all taps'
// loads are issued back to back; with 16-byte accesses on a 16-bit type the input is read through a buffer
// descriptor and a padding tap simply gets an out-of-range offset (the hardware returns zeros), so there is
// no branch between the loads.
template <typename T, int V, int KS>
__global__ __launch_bounds__(256) void dwconv_kernel(DwConvArgs a, long total)
{
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    // tensors hold fewer than 2^30 elements, so 32-bit index arithmetic suffices (64-bit division is slow)
    const unsigned cv = (unsigned)(a.C / V), ui = (unsigned)idx;
    const int c = (int)(ui % cv) * V;
    const unsigned m = ui / cv;
    const int ow = (int)(m % (unsigned)a.Wo);
    const unsigned mh = m / (unsigned)a.Wo;
    const int oh = (int)(mh % (unsigned)a.Ho);
    const int b = (int)(mh / (unsigned)a.Ho);
    const T *x = (const T *)a.x, *w = (const T *)a.w;
    float acc[V];
    if (a.bias) Pack<T, V>::load((const T *)a.bias + c, acc);
    else
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = 0.0f;
    if constexpr (KS > 0 && V == 8 && sizeof(T) == 2) {
        const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, (int)((unsigned)a.B * a.H * a.W * a.C * 2u), 0x00020000);
        typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
        u32x4 xq[KS * KS];
        uint4 wq[KS * KS];
#pragma unroll
        for (int t = 0; t < KS * KS; ++t) {
            const int ih = oh * a.stride - a.pad + t / KS, iw = ow * a.stride - a.pad + t % KS;
            const bool ok = (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
            const unsigned off = ok ? (unsigned)(((b * a.H + ih) * a.W + iw) * a.C + c) * 2u : 0xffffffffu;
            xq[t] = __builtin_amdgcn_raw_buffer_load_b128(rx, off, 0, 0);
            wq[t] = *reinterpret_cast<const uint4 *>(w + (long)t * a.C + c);
        }
#pragma unroll
        for (int t = 0; t < KS * KS; ++t) {
            const uint32_t xs[4] = {xq[t].x, xq[t].y, xq[t].z, xq[t].w}, ws[4] = {wq[t].x, wq[t].y, wq[t].z, wq[t].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[2 * i] = fmaf(Cvt<T>::from_bits(xs[i] & 0xffffu), Cvt<T>::from_bits(ws[i] & 0xffffu), acc[2 * i]);
                acc[2 * i + 1] = fmaf(Cvt<T>::from_bits(xs[i] >> 16), Cvt<T>::from_bits(ws[i] >> 16), acc[2 * i + 1]);
            }
        }
    } else {
        for (int kh = 0; kh < a.KH; ++kh) {
            const int ih = oh * a.stride - a.pad + kh;
            if ((unsigned)ih >= (unsigned)a.H) continue;
            for (int kw = 0; kw < a.KW; ++kw) {
                const int iw = ow * a.stride - a.pad + kw;
                if ((unsigned)iw >= (unsigned)a.W) continue;
                float xv[V], wv[V];
                Pack<T, V>::load(x + (((long)b * a.H + ih) * a.W + iw) * a.C + c, xv);
                Pack<T, V>::load(w + (long)(kh * a.KW + kw) * a.C + c, wv);
#pragma unroll
                for (int i = 0; i < V; ++i) acc[i] = fmaf(xv[i], wv[i], acc[i]);
            }
        }
    }
    const long off = (long)m * a.C + c;
    if (a.res) {
        float rv[V];
        Pack<T, V>::load((const T *)a.res + off, rv);
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] += rv[i];
    }
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = apply_act(a.act, acc[i]);
    Pack<T, V>::store((T *)a.y + off, acc);
}

// 3x3 depthwise, 16-bit type, 8 channels x PW consecutive output pixels of one row per thread.  The one-pixel kernel
// above spends most of its time unpacking: per output element it converts 9 inputs and 9 weights for 9 FMAs and is
// bound by the vector ALU, not by memory.  Here a weight is unpacked once per thread and an input column once per
// row, and each serves up to PW (weights) or 3 (inputs, stride 1) outputs: about 2.5 times fewer instructions per
// output and a third to a half of the load instructions.  Loads of padding pixels use an out-of-range offset.
template <typename T, int PW, int STRIDE>
__global__ __launch_bounds__(256) void dwconv3_row_kernel(DwConvArgs a, unsigned total, unsigned wq)
{
    constexpr int COLS = (PW - 1) * STRIDE + 3;
    const unsigned ui = banded_block() * blockDim.x + threadIdx.x;
    if (ui >= total) return;
    const unsigned cv = (unsigned)a.C >> 3;
    const int c = (int)(ui % cv) * 8;
    const unsigned m = ui / cv;
    const int ow0 = (int)(m % wq) * PW;
    const unsigned mh = m / wq;
    const int oh = (int)(mh % (unsigned)a.Ho);
    const int b = (int)(mh / (unsigned)a.Ho);
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, (int)((unsigned)a.B * a.H * a.W * a.C * 2u), 0x00020000);
    const T *w = (const T *)a.w;
    float acc[PW][8];
    {
        float bv[8];
        if (a.bias) Pack<T, 8>::load((const T *)a.bias + c, bv);
        else
#pragma unroll
            for (int i = 0; i < 8; ++i) bv[i] = 0.0f;
#pragma unroll
        for (int p = 0; p < PW; ++p)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[p][i] = bv[i];
    }
    const int iw0 = ow0 * STRIDE - a.pad, ih0 = oh * STRIDE - a.pad;
    // the columns of input row kh+1 are in flight while row kh is multiplied
    u32x4 xq[2][COLS];
    auto load_row = [&](int kh, u32x4 (&q)[COLS]) {
        const int ih = ih0 + kh;
        const bool row_ok = (unsigned)ih < (unsigned)a.H;
#pragma unroll
        for (int j = 0; j < COLS; ++j) {
            const int iw = iw0 + j;
            const bool ok = row_ok && (unsigned)iw < (unsigned)a.W;
            q[j] = __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? (unsigned)(((b * a.H + ih) * a.W + iw) * a.C + c) * 2u : 0xffffffffu, 0, 0);
        }
    };
    load_row(0, xq[0]);
#pragma unroll
    for (int kh = 0; kh < 3; ++kh) {
        if (kh < 2) load_row(kh + 1, xq[(kh + 1) & 1]);
        float wv[3][8];
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) Pack<T, 8>::load(w + (long)(kh * 3 + kw) * a.C + c, wv[kw]);
#pragma unroll
        for (int j = 0; j < COLS; ++j) {
            const u32x4 q = xq[kh & 1][j];
            const uint32_t xs[4] = {q.x, q.y, q.z, q.w};
            float xv[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) { xv[2 * i] = Cvt<T>::from_bits(xs[i] & 0xffffu); xv[2 * i + 1] = Cvt<T>::from_bits(xs[i] >> 16); }
#pragma unroll
            for (int p = 0; p < PW; ++p) {
                const int kw = j - p * STRIDE;          // a constant once the loops are unrolled
                if (kw >= 0 && kw < 3) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc[p][i] = fmaf(xv[i], wv[kw][i], acc[p][i]);
                }
            }
        }
    }
#pragma unroll
    for (int p = 0; p < PW; ++p) {
        const int ow = ow0 + p;
        if (ow < a.Wo) {
            const long off = ((long)(b * a.Ho + oh) * a.Wo + ow) * a.C + c;
            if (a.res) {
                float rv[8];
                Pack<T, 8>::load((const T *)a.res + off, rv);
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[p][i] += rv[i];
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[p][i] = apply_act(a.act, acc[p][i]);
            Pack<T, 8>::store((T *)a.y + off, acc[p]);
        }
    }
}

// The same for stride-1 layers tall enough to give every compute unit several strips: a thread owns 2 output
// columns x `ph` output rows of 8 channels and walks down its strip.  An input row is then loaded once per strip
// instead of once per output row it touches, the weights, the bias and the index arithmetic are paid once per strip,
// and the input row of the next output row is in flight while the current one is multiplied.
// Arithmetic: the kernel was bound by its vector instructions, not by memory (two per multiply-add: unpack a 16-bit
// value, fused multiply-add; 19 instructions per output element with the weights unpacked again for every row).  Now
// two horizontally adjacent taps of one channel go through one v_dot2 (float accumulate of two 16-bit products): when
// an input row arrives, the columns (0,1) and (1,2) of every channel are packed into pairs with v_perm_b32 -- once per
// input row, used by the three output rows that read it -- and the weights are packed the same way, (kw 0, kw 1), once
// per strip; the third tap of a row stays a fused multiply-add.  10 instructions per output element.  That alone
// changed nothing (237 -> 234 us at 192 x 1120 x 1120): with one row of loads in flight per thread the kernel waits for
// memory, and the registers the packed weights freed now hold three input rows in flight instead of one (-> 217 us).
// Three paired rows are live (ring) and three raw rows are on their way (raw); the walk is unrolled by 3 so that
// ring positions are constants.
template <typename T> struct Dot2;
template <> struct Dot2<bf16_t> {
    __device__ static __forceinline__ float run(uint32_t a, uint32_t b, float c)
    {
        typedef __bf16 v2 __attribute__((ext_vector_type(2)));
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(v2, a), __builtin_bit_cast(v2, b), c, false);
    }
};
template <> struct Dot2<f16_t> {
    __device__ static __forceinline__ float run(uint32_t a, uint32_t b, float c)
    {
        typedef _Float16 v2 __attribute__((ext_vector_type(2)));
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(v2, a), __builtin_bit_cast(v2, b), c, false);
    }
};
// (low half of a, low half of b) and (high half of a, high half of b) as 2 x 16 bits, a in the low half of the result
__device__ __forceinline__ uint32_t pair_lo(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t pair_hi(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

template <typename T, int R>
__global__ __launch_bounds__(256, 2) void dwconv3_strip_kernel(DwConvArgs a, unsigned total, unsigned wq, unsigned hq, int ph)
{
    constexpr int PW = 2, COLS = PW + 2;
    const unsigned ui = banded_block() * blockDim.x + threadIdx.x;
    if (ui >= total) return;
    const unsigned cv = (unsigned)a.C >> 3;
    const int c = (int)(ui % cv) * 8;
    const unsigned m = ui / cv;
    const int ow0 = (int)(m % wq) * PW;
    const unsigned mh = m / wq;
    const int oh0 = (int)(mh % hq) * ph;
    const int b = (int)(mh / hq);
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, (int)((unsigned)a.B * a.H * a.W * a.C * 2u), 0x00020000);
    const T *w = (const T *)a.w;
    uint32_t wpair[3][8];                    // (kw 0, kw 1) of every row of the window, per channel
    float wlast[3][8], bv[8];                // kw 2
#pragma unroll
    for (int kh = 0; kh < 3; ++kh) {
        const uint4 q0 = *reinterpret_cast<const uint4 *>(w + (long)(kh * 3 + 0) * a.C + c);
        const uint4 q1 = *reinterpret_cast<const uint4 *>(w + (long)(kh * 3 + 1) * a.C + c);
        const uint4 q2 = *reinterpret_cast<const uint4 *>(w + (long)(kh * 3 + 2) * a.C + c);
        const uint32_t w0[4] = {q0.x, q0.y, q0.z, q0.w}, w1[4] = {q1.x, q1.y, q1.z, q1.w}, w2[4] = {q2.x, q2.y, q2.z, q2.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            wpair[kh][2 * e] = pair_lo(w0[e], w1[e]);
            wpair[kh][2 * e + 1] = pair_hi(w0[e], w1[e]);
            wlast[kh][2 * e] = Cvt<T>::from_bits(w2[e] & 0xffffu);
            wlast[kh][2 * e + 1] = Cvt<T>::from_bits(w2[e] >> 16);
        }
    }
    if (a.bias) Pack<T, 8>::load((const T *)a.bias + c, bv);
    else
#pragma unroll
        for (int i = 0; i < 8; ++i) bv[i] = 0.0f;
    const int iw0 = ow0 - a.pad, ih0 = oh0 - a.pad;
    unsigned col_off[COLS];                  // byte offset of (column, channel) inside an input row, or out of range
#pragma unroll
    for (int j = 0; j < COLS; ++j) col_off[j] = (unsigned)(iw0 + j) < (unsigned)a.W ? (unsigned)((iw0 + j) * a.C + c) * 2u : 0xffffffffu;
    const unsigned row_bytes = (unsigned)(a.W * a.C) * 2u;
    // a ring row: columns (0,1) and (1,2) paired per channel, and columns 2 and 3 as loaded (8 channels in 4 registers)
    struct Row { uint32_t p01[8], p12[8]; u32x4 c2, c3; };
    static_assert(R == 3, "three paired rows are live, three more are on their way");
    u32x4 raw[R][COLS];                      // rows on their way from memory, three rows ahead of the arithmetic
    Row ring[R];                             // the three rows the current output row reads, paired
    auto load_row = [&](int r, u32x4 (&q)[COLS]) {           // input row ih0 + r of the strip
        const int ih = ih0 + r;
        const bool row_ok = (unsigned)ih < (unsigned)a.H;
        const unsigned base = (unsigned)(b * a.H + ih) * row_bytes;
#pragma unroll
        for (int j = 0; j < COLS; ++j)
            q[j] = __builtin_amdgcn_raw_buffer_load_b128(rx, (row_ok && col_off[j] != 0xffffffffu) ? base + col_off[j] : 0xffffffffu, 0, 0);
    };
    auto take = [&](const u32x4 (&q)[COLS], Row &d) {        // pairs the columns of a row that has arrived
        const uint32_t x0[4] = {q[0].x, q[0].y, q[0].z, q[0].w}, x1[4] = {q[1].x, q[1].y, q[1].z, q[1].w}, x2[4] = {q[2].x, q[2].y, q[2].z, q[2].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            d.p01[2 * e] = pair_lo(x0[e], x1[e]);
            d.p01[2 * e + 1] = pair_hi(x0[e], x1[e]);
            d.p12[2 * e] = pair_lo(x1[e], x2[e]);
            d.p12[2 * e + 1] = pair_hi(x1[e], x2[e]);
        }
        d.c2 = q[2];
        d.c3 = q[3];
    };
    // raw[k] and ring[k] hold rows k (mod 3).  Rows 0..4 are requested up front and rows 0, 1 paired; output row i then
    // pairs row i + 2 and requests row i + 5 into the slot that frees.
    load_row(0, raw[0]); load_row(1, raw[1]); load_row(2, raw[2]);
    take(raw[0], ring[0]); load_row(3, raw[0]);
    take(raw[1], ring[1]); load_row(4, raw[1]);
    for (int i0 = 0; i0 < ph; i0 += R) {
#pragma unroll
        for (int u = 0; u < R; ++u) {
            const int i = i0 + u;                            // output row oh0 + i reads input rows i .. i + 2
            take(raw[(u + 2) % R], ring[(u + 2) % R]);
            load_row(i + 5, raw[(u + 2) % R]);               // beyond the image: zeros
            float acc[PW][8];
#pragma unroll
            for (int p = 0; p < PW; ++p)
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[p][e] = bv[e];
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) {
                const Row &r = ring[(u + kh) % R];
                const uint32_t s2[4] = {r.c2.x, r.c2.y, r.c2.z, r.c2.w}, s3[4] = {r.c3.x, r.c3.y, r.c3.z, r.c3.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    acc[0][e] = Dot2<T>::run(r.p01[e], wpair[kh][e], acc[0][e]);
                    acc[1][e] = Dot2<T>::run(r.p12[e], wpair[kh][e], acc[1][e]);
                    const uint32_t h2 = s2[e >> 1], h3 = s3[e >> 1];
                    acc[0][e] = fmaf(Cvt<T>::from_bits((e & 1) ? h2 >> 16 : h2 & 0xffffu), wlast[kh][e], acc[0][e]);
                    acc[1][e] = fmaf(Cvt<T>::from_bits((e & 1) ? h3 >> 16 : h3 & 0xffffu), wlast[kh][e], acc[1][e]);
                }
            }
            const int oh = oh0 + i;
            if (i < ph && oh < a.Ho) {
#pragma unroll
                for (int p = 0; p < PW; ++p) {
                    const int ow = ow0 + p;
                    if (ow < a.Wo) {
                        const long off = ((long)(b * a.Ho + oh) * a.Wo + ow) * a.C + c;
                        if (a.res) {
                            float rv[8];
                            Pack<T, 8>::load((const T *)a.res + off, rv);
#pragma unroll
                            for (int e = 0; e < 8; ++e) acc[p][e] += rv[e];
                        }
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[p][e] = apply_act(a.act, acc[p][e]);
                        Pack<T, 8>::store((T *)a.y + off, acc[p]);
                    }
                }
            }
        }
    }
}

// ---------------- grouped convolution, channel concatenation, channel shuffle ------------------------------
// (the operators of the second workload family: ResNeXt-, DenseNet- and ShuffleNet-style blocks)
// One thread per output element; the Cin/groups input channels of a tap are contiguous in x and in w, read V at a time.
template <typename T, int V>
__global__ __launch_bounds__(256) void gconv_kernel(GConvArgs a, unsigned total)
{
    const unsigned ui = blockIdx.x * blockDim.x + threadIdx.x;
    if (ui >= total) return;
    const int co = (int)(ui % (unsigned)a.Cout);
    const unsigned m = ui / (unsigned)a.Cout;
    const int ow = (int)(m % (unsigned)a.Wo);
    const unsigned mh = m / (unsigned)a.Wo;
    const int oh = (int)(mh % (unsigned)a.Ho), b = (int)(mh / (unsigned)a.Ho);
    const int cig = a.Cin / a.groups, g = co / (a.Cout / a.groups);
    const T *x = (const T *)a.x, *w = (const T *)a.w + (long)co * a.KH * a.KW * cig;
    float acc = a.bias ? Cvt<T>::load((const T *)a.bias + co) : 0.0f;
    for (int kh = 0; kh < a.KH; ++kh) {
        const int ih = oh * a.stride - a.pad + kh;
        if ((unsigned)ih >= (unsigned)a.H) continue;
        for (int kw = 0; kw < a.KW; ++kw) {
            const int iw = ow * a.stride - a.pad + kw;
            if ((unsigned)iw >= (unsigned)a.W) continue;
            const T *xp = x + (((long)b * a.H + ih) * a.W + iw) * a.Cin + g * cig;
            const T *wp = w + (kh * a.KW + kw) * cig;
            for (int ci = 0; ci < cig; ci += V) {
                float xv[V], wv[V];
                Pack<T, V>::load(xp + ci, xv);
                Pack<T, V>::load(wp + ci, wv);
#pragma unroll
                for (int i = 0; i < V; ++i) acc = fmaf(xv[i], wv[i], acc);
            }
        }
    }
    const long off = (long)m * a.Cout + co;
    if (a.res) acc += Cvt<T>::load((const T *)a.res + off);
    Cvt<T>::store((T *)a.y + off, apply_act(a.act, acc));
}

// one thread per V consecutive output channels; c0 and c1 are multiples of V
template <typename T, int V>
__global__ __launch_bounds__(256) void concat_kernel(const T *a, const T *b, T *y, int c0, int c1, long total)
{
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const unsigned cv = (unsigned)(c0 + c1) / V, ui = (unsigned)idx;
    const int c = (int)(ui % cv) * V;
    const long m = ui / cv;
    float v[V];
    if (c < c0) Pack<T, V>::load(a + m * c0 + c, v);
    else Pack<T, V>::load(b + m * c1 + (c - c0), v);
    Pack<T, V>::store(y + m * (c0 + c1) + c, v);
}

// y[m][0 .. c) = x[m][:] where y's rows are ld channels apart: the first operand of a concatenation done in place
// (c and ld multiples of 8, 16-bit types)
template <typename T>
__global__ __launch_bounds__(256) void chancopy_kernel(const T *x, T *y, int c, int ld, long total)
{
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const unsigned cv = (unsigned)c / 8, ui = (unsigned)idx;
    const unsigned j = (ui % cv) * 8;
    const long m = ui / cv;
    *reinterpret_cast<uint4 *>(y + m * ld + j) = *reinterpret_cast<const uint4 *>(x + m * c + j);
}

template <typename T>
__global__ __launch_bounds__(256) void shuffle_kernel(const T *x, T *y, int c, int groups, long total)
{
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const unsigned ui = (unsigned)idx, j = ui % (unsigned)c;
    const long m = ui / (unsigned)c;
    y[idx] = x[m * c + (j % (unsigned)groups) * (unsigned)(c / groups) + j / (unsigned)groups];
}

// ---------------- max pooling ---------------------------------------------------------------------------
// Window coordinates are clamped into the image instead of skipped: a clamped tap re-reads a pixel that is
// already inside the window (2*pad <= window is checked at load), so the maximum is unchanged and the loads
// need no branch.  KS > 0 fixes the (square) window at compile time.
template <typename T, int V, int KS>
__global__ __launch_bounds__(256) void maxpool_kernel(PoolArgs a, long total)
{
    const long idx = (long)banded_block() * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    // tensors hold fewer than 2^30 elements, so 32-bit index arithmetic suffices (64-bit division is slow)
    const unsigned cv = (unsigned)(a.C / V), ui = (unsigned)idx;
    const int c = (int)(ui % cv) * V;
    const unsigned m = ui / cv;
    const int ow = (int)(m % (unsigned)a.Wo);
    const unsigned mh = m / (unsigned)a.Wo;
    const int oh = (int)(mh % (unsigned)a.Ho);
    const int b = (int)(mh / (unsigned)a.Ho);
    const T *x = (const T *)a.x + (long)b * a.H * a.W * a.C + c;
    float best[V];
#pragma unroll
    for (int i = 0; i < V; ++i) best[i] = -INFINITY;
    const int kh_n = KS > 0 ? KS : a.KH, kw_n = KS > 0 ? KS : a.KW;
    const int ih0 = oh * a.stride - a.pad, iw0 = ow * a.stride - a.pad;
#pragma unroll KS > 0 ? KS : 1
    for (int kh = 0; kh < kh_n; ++kh) {
        const int ih = min(max(ih0 + kh, 0), a.H - 1);
#pragma unroll KS > 0 ? KS : 1
        for (int kw = 0; kw < kw_n; ++kw) {
            const int iw = min(max(iw0 + kw, 0), a.W - 1);
            float xv[V];
            Pack<T, V>::load(x + ((long)ih * a.W + iw) * a.C, xv);
#pragma unroll
            for (int i = 0; i < V; ++i) best[i] = fmaxf(best[i], xv[i]);
        }
    }
    Pack<T, V>::store((T *)a.y + (long)m * a.C + c, best);
}

// 3x3 window, stride 2: a thread produces a block of 2 x PW neighbouring outputs.  Their windows span five input rows
// and 2 PW + 1 columns and share the middle ones, so a block of four costs 25 loads instead of 36 (a vertical pair 15
// instead of 18), all independent and in flight together.  Rows and columns are clamped as above; outputs of the
// block that fall outside an odd-sized result are not stored (a clamped row or column that only they would use is
// then never used).  Launched with PW = 1: at 64 x 1792 x 1792 the vertical pair takes 93.5 us, the single-output
// kernel 96.0 and the 2 x 2 block 98.2.
template <typename T, int V, int PW>
__global__ __launch_bounds__(256) void maxpool3s2_block_kernel(PoolArgs a, long total)
{
    const long idx = (long)banded_block() * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const unsigned cv = (unsigned)(a.C / V), ui = (unsigned)idx, hp = (unsigned)(a.Ho + 1) >> 1, wq = (unsigned)(a.Wo + PW - 1) / PW;
    const int c = (int)(ui % cv) * V;
    const unsigned m = ui / cv;
    const int ow0 = (int)(m % wq) * PW;
    const unsigned mh = m / wq;
    const int oh0 = (int)(mh % hp) * 2;
    const int b = (int)(mh / hp);
    const T *x = (const T *)a.x + (long)b * a.H * a.W * a.C + c;
    const int ih0 = oh0 * 2 - a.pad, iw0 = ow0 * 2 - a.pad;
    constexpr int NC = 2 * PW + 1;
    float xv[5][NC][V];
#pragma unroll
    for (int r = 0; r < 5; ++r) {
        const int ih = min(max(ih0 + r, 0), a.H - 1);
#pragma unroll
        for (int q = 0; q < NC; ++q) {
            const int iw = min(max(iw0 + q, 0), a.W - 1);
            Pack<T, V>::load(x + ((long)ih * a.W + iw) * a.C, xv[r][q]);
        }
    }
    T *y = (T *)a.y + (((long)b * a.Ho + oh0) * a.Wo + ow0) * a.C + c;
#pragma unroll
    for (int j = 0; j < PW; ++j) {
        float row[5][V];
#pragma unroll
        for (int r = 0; r < 5; ++r)
#pragma unroll
            for (int i = 0; i < V; ++i) row[r][i] = fmaxf(fmaxf(xv[r][2 * j][i], xv[r][2 * j + 1][i]), xv[r][2 * j + 2][i]);
        float o0[V], o1[V];
#pragma unroll
        for (int i = 0; i < V; ++i) {
            o0[i] = fmaxf(fmaxf(row[0][i], row[1][i]), row[2][i]);
            o1[i] = fmaxf(fmaxf(row[2][i], row[3][i]), row[4][i]);
        }
        if (ow0 + j < a.Wo) {
            Pack<T, V>::store(y + (long)j * a.C, o0);
            if (oh0 + 1 < a.Ho) Pack<T, V>::store(y + ((long)a.Wo + j) * a.C, o1);
        }
    }
}

// ---------------- global average pooling: block = 32 channel chunks x 8 row slices -------------------------
// grid = (channel blocks, B, hw_parts).  With hw_parts == 1 the block finishes its channels; otherwise it
// writes the float sums of its share of the rows to part_out[b][part][C] and gap_finish_kernel adds the parts.
template <typename T, int V>
__global__ __launch_bounds__(256) void gap_kernel(const T *x, T *y, float *y32, float *part_out, int HW, int C)
{
    __shared__ float part[8][32][V];
    const int b = blockIdx.y;
    const int lane_c = threadIdx.x & 31, slice = threadIdx.x >> 5;
    const int c = (blockIdx.x * 32 + lane_c) * V;
    const int parts = gridDim.z;
    const int per = (HW + parts - 1) / parts;
    const int r0 = blockIdx.z * per, r1 = min(HW, r0 + per);
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.0f;
    if (c < C) {
        // four rows in flight per thread (independent loads, one running sum: the order of additions is fixed)
        int r = r0 + slice;
        for (; r + 24 < r1; r += 32) {
            float xv[4][V];
#pragma unroll
            for (int u = 0; u < 4; ++u) Pack<T, V>::load(x + ((long)b * HW + r + 8 * u) * C + c, xv[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int i = 0; i < V; ++i) acc[i] += xv[u][i];
        }
        for (; r < r1; r += 8) {
            float xv[V];
            Pack<T, V>::load(x + ((long)b * HW + r) * C + c, xv);
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] += xv[i];
        }
    }
#pragma unroll
    for (int i = 0; i < V; ++i) part[slice][lane_c][i] = acc[i];
    __syncthreads();
    if (slice == 0 && c < C) {
        float o[V];
#pragma unroll
        for (int i = 0; i < V; ++i) {
            float s = 0.0f;
#pragma unroll
            for (int j = 0; j < 8; ++j) s += part[j][lane_c][i];
            o[i] = s;
        }
        if (parts > 1) {
#pragma unroll
            for (int i = 0; i < V; ++i) part_out[((long)b * parts + blockIdx.z) * C + c + i] = o[i];
            return;
        }
        const float inv = 1.0f / (float)HW;
#pragma unroll
        for (int i = 0; i < V; ++i) o[i] *= inv;
        if (y32) {
#pragma unroll
            for (int i = 0; i < V; ++i) y32[(long)b * C + c + i] = o[i];
        } else {
            Pack<T, V>::store(y + (long)b * C + c, o);
        }
    }
}
template <typename T>
__global__ __launch_bounds__(256) void gap_finish_kernel(const float *part_in, T *y, float *y32, int parts, int HW, int C, long total)
{
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;     // over B*C
    if (idx >= total) return;
    const long b = (unsigned)idx / (unsigned)C, c = (unsigned)idx % (unsigned)C;
    float s = 0.0f;
    for (int p = 0; p < parts; ++p) s += part_in[(b * parts + p) * C + c];
    s *= 1.0f / (float)HW;
    if (y32) y32[idx] = s;
    else Cvt<T>::store(y + idx, s);
}

// ---------------- row kernels: LPR lanes per row, the row lives in registers ----------------------------------
// A row is shared by LPR lanes of a wavefront (16, 32 or 64), which therefore carries 64 / LPR rows at a time; lane l of
// a row's group owns chunks l, l + LPR, ... (V elements each), NCH chunks per lane at most.  Narrow rows on a whole
// wavefront leave lanes idle and very few bytes in flight per wavefront (a 384-element row is 48 chunks of 16 bytes: a
// quarter of the lanes had nothing to do and a wavefront had 768 bytes on their way); with 16 lanes per row every lane
// works, the reductions take 4 exchanges instead of 6, and a wavefront has four rows in flight.
template <typename T, int V, int NCH, int LPR, bool SOFTMAX>
__global__ __launch_bounds__(256) void row_kernel(RowArgs a)
{
    constexpr int RPW = 64 / LPR;                     // rows per wavefront
    const int lane = threadIdx.x & 63, sub = lane & (LPR - 1);
    const long row = ((long)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW + lane / LPR;
    const bool live = row < a.rows;                   // lanes of rows past the end still take part in the exchanges
    const int nchunk = a.width / V;
    const T *x = (const T *)a.x + (live ? row : 0) * a.width;
    const T *r = a.res ? (const T *)a.res + (live ? row : 0) * a.width : nullptr;
    float v[NCH][V];
    float s = 0.0f, mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        const int ch = sub + j * LPR;
        if (ch < nchunk) Pack<T, V>::load(x + ch * V, v[j]);
    }
    if (r) {
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const int ch = sub + j * LPR;
            if (ch < nchunk) {
                float rv[V];
                Pack<T, V>::load(r + ch * V, rv);
#pragma unroll
                for (int i = 0; i < V; ++i) v[j][i] += rv[i];
            }
        }
    }
#pragma unroll
    for (int j = 0; j < NCH; ++j)
        if (sub + j * LPR < nchunk)
#pragma unroll
            for (int i = 0; i < V; ++i) { s += v[j][i]; mx = fmaxf(mx, v[j][i]); }
    float scale, shift;   // y = (v - shift) * scale  (LayerNorm)   |   y = exp(v - shift) * scale (softmax)
    if (SOFTMAX) {
        mx = group_max<LPR>(mx);
        float es = 0.0f;
#pragma unroll
        for (int j = 0; j < NCH; ++j)
            if (sub + j * LPR < nchunk)
#pragma unroll
                for (int i = 0; i < V; ++i) { v[j][i] = __expf(v[j][i] - mx); es += v[j][i]; }
        es = group_sum<LPR>(es);
        scale = 1.0f / es;
        shift = 0.0f;
    } else {
        const float mean = group_sum<LPR>(s) / (float)a.width;
        float q = 0.0f;
#pragma unroll
        for (int j = 0; j < NCH; ++j)
            if (sub + j * LPR < nchunk)
#pragma unroll
                for (int i = 0; i < V; ++i) { const float d = v[j][i] - mean; q += d * d; }
        const float var = group_sum<LPR>(q) / (float)a.width;
        scale = rsqrtf(var + a.eps);
        shift = mean;
    }
    if (!live) return;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        const int ch = sub + j * LPR;
        if (ch < nchunk) {
            float o[V];
#pragma unroll
            for (int i = 0; i < V; ++i) o[i] = (v[j][i] - shift) * scale;
            if (!SOFTMAX) {
                if (a.gamma) {
                    float g[V];
                    Pack<T, V>::load((const T *)a.gamma + ch * V, g);
#pragma unroll
                    for (int i = 0; i < V; ++i) o[i] *= g[i];
                }
                if (a.beta) {
                    float be[V];
                    Pack<T, V>::load((const T *)a.beta + ch * V, be);
#pragma unroll
                    for (int i = 0; i < V; ++i) o[i] += be[i];
                }
            }
            if (a.y32) {
#pragma unroll
                for (int i = 0; i < V; ++i) a.y32[row * a.width + ch * V + i] = o[i];
            } else {
                Pack<T, V>::store((T *)a.y + row * a.width + ch * V, o);
            }
        }
    }
}

// ---------------- element-wise epilogue ---------------------------------------------------------------------
// A thread handles U vectors, `stride` vectors apart (so that a wavefront's accesses stay contiguous for every one of
// them), and issues all of its loads before the arithmetic of the first.
template <typename T, int V, int U>
__global__ __launch_bounds__(256) void eltwise_kernel(EltArgs a, long total, long stride)
{
    const long idx0 = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const unsigned cv = (unsigned)(a.width / V);
    float v[U][V], t[U][V];
    long off[U];
    int c[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const long idx = idx0 + u * stride;
        ok[u] = idx < total;
        const unsigned ui = (unsigned)(ok[u] ? idx : 0);
        c[u] = (int)(ui % cv) * V;
        off[u] = (long)(ui / cv) * a.width + c[u];
        if (ok[u]) Pack<T, V>::load((const T *)a.x + off[u], v[u]);
    }
    if (a.res) {
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (ok[u]) {
                Pack<T, V>::load((const T *)a.res + off[u], t[u]);
#pragma unroll
                for (int i = 0; i < V; ++i) v[u][i] += t[u][i];
            }
    }
    if (a.bias) {
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (ok[u]) {
                Pack<T, V>::load((const T *)a.bias + c[u], t[u]);
#pragma unroll
                for (int i = 0; i < V; ++i) v[u][i] += t[u][i];
            }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (!ok[u]) continue;
#pragma unroll
        for (int i = 0; i < V; ++i) v[u][i] = apply_act(a.act, v[u][i]);
        if (a.y32) {
#pragma unroll
            for (int i = 0; i < V; ++i) a.y32[off[u] + i] = v[u][i];
        } else {
            Pack<T, V>::store((T *)a.y + off[u], v[u]);
        }
    }
}

// ---------------- embedding gather ----------------------------------------------------------------------------
template <typename T, int V>
__global__ __launch_bounds__(256) void embed_kernel(EmbedArgs a, long total)
{
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const unsigned cv = (unsigned)(a.Hd / V), ui = (unsigned)idx;
    const int c = (int)(ui % cv) * V;
    const long tokn = ui / cv;
    const int s = (int)((unsigned)tokn % (unsigned)a.S);
    int id = a.ids[tokn];
    id = id < 0 ? 0 : (id >= a.vocab ? a.vocab - 1 : id);     // out-of-range ids are clamped, never read out of bounds
    float t[V], p[V], ty[V], o[V];
    Pack<T, V>::load((const T *)a.tok + (long)id * a.Hd + c, t);
    Pack<T, V>::load((const T *)a.pos + (long)s * a.Hd + c, p);
    Pack<T, V>::load((const T *)a.typ + c, ty);
#pragma unroll
    for (int i = 0; i < V; ++i) o[i] = t[i] + p[i] + ty[i];
    Pack<T, V>::store((T *)a.y + tokn * a.Hd + c, o);
}

// ---------------- boundary layout conversions -------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void nchw_to_nhwc_kernel(const T *x, T *y, int C, int HW, int Cp, long total)
{
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;   // over B*HW*Cp
    if (idx >= total) return;
    const unsigned ui = (unsigned)idx;
    const int c = (int)(ui % (unsigned)Cp);
    const unsigned bp = ui / (unsigned)Cp;
    const long b = bp / (unsigned)HW, pix = bp % (unsigned)HW;
    T v;
    if (c < C) v = x[(b * C + c) * HW + pix];
    else Cvt<T>::store(&v, 0.0f);
    y[idx] = v;
}
template <typename T>
__global__ __launch_bounds__(256) void nhwc_to_nchw_f32_kernel(const T *x, float *y, int C, int HW, long total)
{
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;   // over B*C*HW (output order)
    if (idx >= total) return;
    const unsigned ui = (unsigned)idx;
    const int pix = (int)(ui % (unsigned)HW);
    const unsigned bc = ui / (unsigned)HW;
    const long b = bc / (unsigned)C, c = bc % (unsigned)C;
    y[idx] = Cvt<T>::load(x + (b * HW + pix) * C + c);
}
template <typename T>
__global__ __launch_bounds__(256) void to_f32_kernel(const T *x, float *y, long n)
{
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < n) y[idx] = Cvt<T>::load(x + idx);
}

// ---------------- diagnostics --------------------------------------------------------------------------------------
__global__ void probe_kernel(uint32_t *out)
{
    // HW_ID (hwreg 4): cu_id bits 8..11, sh_id bit 12, se_id bits 13..15; XCC_ID (hwreg 20): bits 0..3
    const uint32_t hw = __builtin_amdgcn_s_getreg(4 | (0 << 6) | (31 << 11));
    const uint32_t xcc = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11));
    if (threadIdx.x == 0) {
        const uint32_t cu = (hw >> 8) & 0xf, sh = (hw >> 12) & 1, se = (hw >> 13) & 7;
        out[blockIdx.x] = (xcc << 16) | (se << 8) | (sh << 4) | cu;
    }
    // stay resident long enough that workgroups spread over every enabled CU
    const long long t0 = wall_clock64();
    while (wall_clock64() - t0 < 20000) { }
}
__global__ void tick_kernel(uint32_t *p)
{
    if (threadIdx.x == 0) p[0] = p[0] + 1u;
}
__global__ void fill_u32_kernel(uint32_t *p, uint32_t v, long n)
{
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < n) p[idx] = v;
}

}  // namespace

hipError_t launch_conv_f32(const ConvF32Args &a, hipStream_t s)
{
    const long total = (long)a.B * a.Ho * a.Wo * a.Cout;
    hipLaunchKernelGGL(conv_f32_kernel, dim3(blocks_for(total, 256)), dim3(256), 0, s, a, total);
    return hipGetLastError();
}

// Large 3x3 layers of a 16-bit type run four output pixels per thread, as long as that still leaves four
// workgroups for every compute unit.
int dwconv_pixels_per_thread(const DwConvArgs &a, int n_cu)
{
    if (a.dtype == DT_F32 || a.KH != 3 || a.KW != 3 || (a.C & 7) != 0 || (a.stride != 1 && a.stride != 2)) return 1;
    const long total = (long)a.B * a.Ho * ((a.Wo + 3) / 4) * (a.C / 8);
    return (total >= 4L * n_cu * 256 && total < (1L << 31)) ? 4 : 1;
}

// Output rows per thread of the strip kernel (a multiple of its ring size, 3), or 0 when the layer is not a stride-1
// 3x3 one with at least 4 workgroups of strips per compute unit: the tallest of 24, 18, 12, 9 that leaves that many.
int dwconv_strip_rows(const DwConvArgs &a, int n_cu)
{
    if (dwconv_pixels_per_thread(a, n_cu) != 4 || a.stride != 1) return 0;
    for (int ph : {24, 18, 12, 9}) {
        const long strips = (long)a.B * ((a.Ho + ph - 1) / ph) * ((a.Wo + 1) / 2) * (a.C / 8);
        if (strips >= 4L * n_cu * 256) return ph;
    }
    return 0;
}

hipError_t launch_dwconv(const DwConvArgs &a, int n_cu, hipStream_t s)
{
    if (dwconv_pixels_per_thread(a, n_cu) == 4) {
        const unsigned wq = (unsigned)(a.Wo + 3) / 4;
        const int ph = dwconv_strip_rows(a, n_cu);
        if (ph) {                                            // tall stride-1 images: 2 x ph output pixels per thread
            const unsigned hq = (unsigned)(a.Ho + ph - 1) / ph, wq2 = (unsigned)(a.Wo + 1) / 2;
            const long strips = (long)a.B * hq * wq2 * (a.C / 8);
            const dim3 grid(banded_blocks_for(strips, 256));
            if (a.dtype == DT_BF16) hipLaunchKernelGGL((dwconv3_strip_kernel<bf16_t, 3>), grid, dim3(256), 0, s, a, (unsigned)strips, wq2, hq, ph);
            else hipLaunchKernelGGL((dwconv3_strip_kernel<f16_t, 3>), grid, dim3(256), 0, s, a, (unsigned)strips, wq2, hq, ph);
            return hipGetLastError();
        }
        const long total = (long)a.B * a.Ho * wq * (a.C / 8);
        {
            const dim3 grid(banded_blocks_for(total, 256));
#define ROW(T)                                                                                                          \
    if (a.stride == 1) hipLaunchKernelGGL((dwconv3_row_kernel<T, 4, 1>), grid, dim3(256), 0, s, a, (unsigned)total, wq); \
    else hipLaunchKernelGGL((dwconv3_row_kernel<T, 4, 2>), grid, dim3(256), 0, s, a, (unsigned)total, wq);
            if (a.dtype == DT_BF16) { ROW(bf16_t) } else { ROW(f16_t) }
#undef ROW
            return hipGetLastError();
        }
    }
#define CALL(T, V)                                                                                              \
    {                                                                                                           \
        const long total = (long)a.B * a.Ho * a.Wo * (a.C / V);                                                 \
        const dim3 grid(blocks_for(total, 256));                                                                \
        if (a.KH == 3 && a.KW == 3) hipLaunchKernelGGL((dwconv_kernel<T, V, 3>), grid, dim3(256), 0, s, a, total); \
        else hipLaunchKernelGGL((dwconv_kernel<T, V, 0>), grid, dim3(256), 0, s, a, total);                     \
    }
    ECLIP_DISPATCH(a.dtype, a.C, CALL);
#undef CALL
    return hipGetLastError();
}

hipError_t launch_maxpool(const PoolArgs &a, int, hipStream_t s)
{
#define CALL(T, V)                                                                                               \
    {                                                                                                            \
        const long total = (long)a.B * a.Ho * a.Wo * (a.C / V);                                                  \
        const dim3 grid(banded_blocks_for(total, 256));                                                          \
        if (a.KH == 3 && a.KW == 3 && a.stride == 2 && V > 1) {                                                  \
            const long blocks = (long)a.B * ((a.Ho + 1) / 2) * a.Wo * (a.C / V);                                 \
            hipLaunchKernelGGL((maxpool3s2_block_kernel<T, V, 1>), dim3(banded_blocks_for(blocks, 256)), dim3(256), 0, s, a, blocks); \
        } else if (a.KH == 3 && a.KW == 3) hipLaunchKernelGGL((maxpool_kernel<T, V, 3>), grid, dim3(256), 0, s, a, total); \
        else if (a.KH == 2 && a.KW == 2) hipLaunchKernelGGL((maxpool_kernel<T, V, 2>), grid, dim3(256), 0, s, a, total); \
        else hipLaunchKernelGGL((maxpool_kernel<T, V, 0>), grid, dim3(256), 0, s, a, total);                     \
    }
    ECLIP_DISPATCH(a.dtype, a.C, CALL);
#undef CALL
    return hipGetLastError();
}

hipError_t launch_gconv(const GConvArgs &a, int, hipStream_t s)
{
    const long total = (long)a.B * a.Ho * a.Wo * a.Cout;
    if (total >= (1L << 31)) return hipErrorInvalidValue;
    const int cig = a.Cin / a.groups;
    const dim3 grid(blocks_for(total, 256));
#define G(T)                                                                                               \
    if (cig % 8 == 0) hipLaunchKernelGGL((gconv_kernel<T, 8>), grid, dim3(256), 0, s, a, (unsigned)total);      \
    else if (cig % 4 == 0) hipLaunchKernelGGL((gconv_kernel<T, 4>), grid, dim3(256), 0, s, a, (unsigned)total); \
    else hipLaunchKernelGGL((gconv_kernel<T, 1>), grid, dim3(256), 0, s, a, (unsigned)total);
    if (a.dtype == DT_BF16) { G(bf16_t) } else if (a.dtype == DT_F16) { G(f16_t) } else return hipErrorInvalidValue;
#undef G
    return hipGetLastError();
}

hipError_t launch_concat(const void *a, const void *b, void *y, long rows, int c0, int c1, int dtype, hipStream_t s)
{
    if (rows * (c0 + c1) >= (1L << 31)) return hipErrorInvalidValue;
    const int unit = dtype == DT_F32 ? 4 : 8;
    const bool vec = c0 % unit == 0 && c1 % unit == 0;
#define CC(T, V)                                                                                                       \
    {                                                                                                                  \
        const long total = rows * ((c0 + c1) / V);                                                                     \
        hipLaunchKernelGGL((concat_kernel<T, V>), dim3(blocks_for(total, 256)), dim3(256), 0, s, (const T *)a, (const T *)b, (T *)y, c0, c1, total); \
    }
    if (dtype == DT_F32) { if (vec) CC(float, 4) else CC(float, 1) }
    else if (dtype == DT_BF16) { if (vec) CC(bf16_t, 8) else CC(bf16_t, 1) }
    else { if (vec) CC(f16_t, 8) else CC(f16_t, 1) }
#undef CC
    return hipGetLastError();
}

hipError_t launch_chancopy(const void *x, void *y, long rows, int c, int ld, int dtype, hipStream_t s)
{
    if (dtype == DT_F32 || c % 8 || ld % 8 || ld < c || rows * (long)ld >= (1L << 31)) return hipErrorInvalidValue;
    const long total = rows * (c / 8);
    hipLaunchKernelGGL((chancopy_kernel<uint16_t>), dim3(blocks_for(total, 256)), dim3(256), 0, s, (const uint16_t *)x, (uint16_t *)y, c, ld, total);
    return hipGetLastError();
}

hipError_t launch_shuffle(const void *x, void *y, long rows, int c, int groups, int dtype, hipStream_t s)
{
    const long total = rows * c;
    if (total >= (1L << 31)) return hipErrorInvalidValue;
    const dim3 grid(blocks_for(total, 256));
    if (dtype == DT_F32) hipLaunchKernelGGL((shuffle_kernel<uint32_t>), grid, dim3(256), 0, s, (const uint32_t *)x, (uint32_t *)y, c, groups, total);
    else hipLaunchKernelGGL((shuffle_kernel<uint16_t>), grid, dim3(256), 0, s, (const uint16_t *)x, (uint16_t *)y, c, groups, total);
    return hipGetLastError();
}

int gap_parts(int B, int HW, int C, int n_cu)
{
    // enough workgroups to cover the CUs twice, at least 64 rows per part
    const long base = (long)B * ((C + 255) / 256);
    long parts = (2L * n_cu + base - 1) / base;
    const long cap = HW / 64 > 0 ? HW / 64 : 1;
    if (parts > cap) parts = cap;
    if (parts > 64) parts = 64;
    return parts < 1 ? 1 : (int)parts;
}

hipError_t launch_gap(const void *x, void *y, float *y32, float *ws, size_t ws_floats, int B, int HW, int C, int dtype, int n_cu,
                      hipStream_t s, uint32_t *n_launched)
{
    int parts = gap_parts(B, HW, C, n_cu);
    if ((size_t)B * parts * C > ws_floats) parts = 1;
    if (n_launched) *n_launched += parts > 1 ? 2 : 1;
#define CALL(T, V)                                                                                                     \
    {                                                                                                                  \
        const dim3 grid(blocks_for(C / V, 32), (unsigned)B, (unsigned)parts);                                          \
        hipLaunchKernelGGL((gap_kernel<T, V>), grid, dim3(256), 0, s, (const T *)x, (T *)y, y32, ws, HW, C);           \
        if (parts > 1) {                                                                                               \
            const long total = (long)B * C;                                                                            \
            hipLaunchKernelGGL((gap_finish_kernel<T>), dim3(blocks_for(total, 256)), dim3(256), 0, s, ws, (T *)y, y32, parts, HW, C, total); \
        }                                                                                                              \
    }
    ECLIP_DISPATCH(dtype, C, CALL);
#undef CALL
    return hipGetLastError();
}

// ---------------- global average pool + classifier in one launch ------------------------------------------------
// y[b][n] = act(bias[n] + sum_c mean_hw(x[b][hw][c]) * w[n][c]) for a small batch.  Every kernel costs a few
// microseconds whatever it does, and after the pooling a classifier at batch 1 is a matrix-vector product: one launch
// saves one of the two.  A workgroup first pools all C channels into LDS (float; each thread sums a share of the
// pixels of one 16-byte channel chunk), then each of its 4 wavefronts takes one block of 16 outputs and walks the
// weights in their blocked layout (1 KB blocks of 16 outputs x 32 channels, lane l = output l & 15, channels
// 8 (l >> 4) .. +7), so that every weight load of a wavefront is one contiguous kilobyte.  The pooled vector is read
// once per workgroup, which is what limits the form to moderate C x HW (the caller decides).
template <typename T>
__global__ __launch_bounds__(256) void gapfc_kernel(const T *x, const uint4 *wb, const T *bias, T *y, float *y32, int HW, int C, int N,
                                                    int KB, int act)
{
    extern __shared__ __attribute__((aligned(16))) float gsm[];       // pooled[KB * 32], then part[parts][C]
    float *pooled = gsm, *part = gsm + KB * 32;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.y;
    const int cv = C >> 3, parts = 256 / cv;                           // C % 8 == 0 and C <= 2048 (checked by the caller)
    if (tid < parts * cv) {
        const int chunk = tid % cv, pt = tid / cv;
        const T *src = x + ((long)b * HW) * C + chunk * 8;
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
        int px = pt;
        for (; px + 3 * parts < HW; px += 4 * parts) {                 // four loads in flight
            float v[4][8];
#pragma unroll
            for (int u = 0; u < 4; ++u) Pack<T, 8>::load(src + (long)(px + u * parts) * C, v[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] += v[u][e];
        }
        for (; px < HW; px += parts) {
            float v[8];
            Pack<T, 8>::load(src + (long)px * C, v);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += v[e];
        }
        float *dst = part + pt * C + chunk * 8;
        *reinterpret_cast<float4 *>(dst) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        *reinterpret_cast<float4 *>(dst + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
    __syncthreads();
    const float inv = 1.0f / (float)HW;
    for (int c = tid; c < KB * 32; c += 256) {
        float sum = 0.0f;
        if (c < C)
            for (int pt = 0; pt < parts; ++pt) sum += part[pt * C + c];
        pooled[c] = sum * inv;                                         // zero beyond C: the weight blocks are padded too
    }
    __syncthreads();
    const int nb = blockIdx.x * 4 + wave;
    if (nb * 16 >= N) return;
    const uint4 *wrow = wb + (long)nb * KB * 64 + lane;
    const float *pv = pooled + (lane >> 4) * 8;
    float acc = 0.0f;
    int kb = 0;
    for (; kb + 4 <= KB; kb += 4) {
        uint4 q[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) q[u] = wrow[(kb + u) * 64];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t ws4[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
            const float4 p0 = *reinterpret_cast<const float4 *>(pv + (kb + u) * 32), p1 = *reinterpret_cast<const float4 *>(pv + (kb + u) * 32 + 4);
            const float pe[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc = fmaf(Cvt<T>::from_bits(ws4[e] & 0xffffu), pe[2 * e], acc);
                acc = fmaf(Cvt<T>::from_bits(ws4[e] >> 16), pe[2 * e + 1], acc);
            }
        }
    }
    for (; kb < KB; ++kb) {
        const uint4 q = wrow[kb * 64];
        const uint32_t ws4[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc = fmaf(Cvt<T>::from_bits(ws4[e] & 0xffffu), pv[kb * 32 + 2 * e], acc);
            acc = fmaf(Cvt<T>::from_bits(ws4[e] >> 16), pv[kb * 32 + 2 * e + 1], acc);
        }
    }
    acc += __shfl_xor(acc, 16, 64);
    acc += __shfl_xor(acc, 32, 64);
    const int n = nb * 16 + lane;
    if (lane < 16 && n < N) {
        float v = acc + (bias ? Cvt<T>::load(bias + n) : 0.0f);
        v = apply_act(act, v);
        if (y32) y32[(long)b * N + n] = v;
        else Cvt<T>::store(y + (long)b * N + n, v);
    }
}

bool gapfc_supported(int B, int HW, int C, int dtype)
{
    // the pooled tensor is re-read by every workgroup and the weights by every batch item: small cases only
    return (dtype == DT_BF16 || dtype == DT_F16) && B <= 8 && C % 8 == 0 && C >= 8 && C <= 2048 && (long)HW * C <= 64 * 1024;
}

hipError_t launch_gapfc(const void *x, const void *w_blocked, const void *bias, void *y, float *y32, int B, int HW, int C, int N, int act,
                        int dtype, hipStream_t s)
{
    if (!gapfc_supported(B, HW, C, dtype)) return hipErrorInvalidValue;
    const int KB = (C + 31) / 32, NB = (N + 15) / 16, parts = 256 / (C / 8);
    const size_t lds = ((size_t)KB * 32 + (size_t)parts * C) * sizeof(float);
    const dim3 grid((unsigned)((NB + 3) / 4), (unsigned)B);
    if (dtype == DT_BF16)
        hipLaunchKernelGGL(gapfc_kernel<bf16_t>, grid, dim3(256), lds, s, (const bf16_t *)x, (const uint4 *)w_blocked, (const bf16_t *)bias, (bf16_t *)y, y32, HW, C, N, KB, act);
    else
        hipLaunchKernelGGL(gapfc_kernel<f16_t>, grid, dim3(256), lds, s, (const f16_t *)x, (const uint4 *)w_blocked, (const f16_t *)bias, (f16_t *)y, y32, HW, C, N, KB, act);
    return hipGetLastError();
}

template <bool SOFTMAX>
static hipError_t launch_row(const RowArgs &a, hipStream_t s)
{
    // rows of up to 48 chunks share a wavefront four at a time (16 lanes each: softmax over 384 keys 62 -> 69 % of the HBM
    // peak); wider rows take a whole wavefront (two rows of 128 chunks per wavefront on 32 lanes each measured slower:
    // LayerNorm over 1024 elements 72 -> 69 %)
#define ROWK(T, V, NCH, LPR) \
    hipLaunchKernelGGL((row_kernel<T, V, NCH, LPR, SOFTMAX>), dim3(blocks_for(a.rows, 4 * (64 / LPR))), dim3(256), 0, s, a)
#define CALL(T, V)                                                                                  \
    {                                                                                               \
        const int nchunk = a.width / V;                                                             \
        if (nchunk <= 16) ROWK(T, V, 1, 16);                                                        \
        else if (nchunk <= 32) ROWK(T, V, 2, 16);                                                   \
        else if (nchunk <= 48) ROWK(T, V, 3, 16);                                                   \
        else if (nchunk <= 128) ROWK(T, V, 2, 64);                                                  \
        else if (nchunk <= 256) ROWK(T, V, 4, 64);                                                  \
        else if (nchunk <= 1024) ROWK(T, V, 16, 64);                                                \
        else return hipErrorInvalidValue;                                                           \
    }
    ECLIP_DISPATCH(a.dtype, a.width, CALL);
#undef CALL
#undef ROWK
    return hipGetLastError();
}
hipError_t launch_layernorm(const RowArgs &a, int, hipStream_t s) { return launch_row<false>(a, s); }
hipError_t launch_softmax(const RowArgs &a, int, hipStream_t s) { return launch_row<true>(a, s); }

hipError_t launch_eltwise(const EltArgs &a, int, hipStream_t s)
{
#define CALL(T, V)                                                                                           \
    {                                                                                                        \
        const long total = a.rows * (a.width / V);                                                           \
        /* one vector per thread: four per thread with all loads issued first measured slower (copy 79 -> 71 % of the HBM peak) */ \
        hipLaunchKernelGGL((eltwise_kernel<T, V, 1>), dim3(blocks_for(total, 256)), dim3(256), 0, s, a, total, 0L); \
    }
    ECLIP_DISPATCH(a.dtype, a.width, CALL);
#undef CALL
    return hipGetLastError();
}

hipError_t launch_embed(const EmbedArgs &a, int, hipStream_t s)
{
#define CALL(T, V)                                                                                         \
    {                                                                                                      \
        const long total = (long)a.B * a.S * (a.Hd / V);                                                   \
        hipLaunchKernelGGL((embed_kernel<T, V>), dim3(blocks_for(total, 256)), dim3(256), 0, s, a, total); \
    }
    ECLIP_DISPATCH(a.dtype, a.Hd, CALL);
#undef CALL
    return hipGetLastError();
}

#define ECLIP_DT(dtype, CALL)                     \
    do {                                          \
        if ((dtype) == DT_F32) { CALL(float); }   \
        else if ((dtype) == DT_BF16) { CALL(bf16_t); } \
        else { CALL(f16_t); }                     \
    } while (0)

hipError_t launch_nchw_to_nhwc(const void *x, void *y, int B, int C, int H, int W, int Cp, int dtype, hipStream_t s)
{
    const long total = (long)B * H * W * Cp;
#define CALL(T) hipLaunchKernelGGL((nchw_to_nhwc_kernel<T>), dim3(blocks_for(total, 256)), dim3(256), 0, s, (const T *)x, (T *)y, C, H * W, Cp, total)
    ECLIP_DT(dtype, CALL);
#undef CALL
    return hipGetLastError();
}
hipError_t launch_nhwc_to_nchw_f32(const void *x, float *y, int B, int C, int H, int W, int dtype, hipStream_t s)
{
    const long total = (long)B * C * H * W;
#define CALL(T) hipLaunchKernelGGL((nhwc_to_nchw_f32_kernel<T>), dim3(blocks_for(total, 256)), dim3(256), 0, s, (const T *)x, y, C, H * W, total)
    ECLIP_DT(dtype, CALL);
#undef CALL
    return hipGetLastError();
}
hipError_t launch_to_f32(const void *x, float *y, long n, int dtype, hipStream_t s)
{
#define CALL(T) hipLaunchKernelGGL((to_f32_kernel<T>), dim3(blocks_for(n, 256)), dim3(256), 0, s, (const T *)x, y, n)
    ECLIP_DT(dtype, CALL);
#undef CALL
    return hipGetLastError();
}

hipError_t launch_probe(uint32_t *out, int n_blocks, hipStream_t s)
{
    hipLaunchKernelGGL(probe_kernel, dim3((unsigned)n_blocks), dim3(64), 0, s, out);
    return hipGetLastError();
}
hipError_t launch_tick(uint32_t *p, hipStream_t s)
{
    hipLaunchKernelGGL(tick_kernel, dim3(1), dim3(64), 0, s, p);
    return hipGetLastError();
}
hipError_t launch_fill_u32(uint32_t *p, uint32_t v, long n, hipStream_t s)
{
    hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, s, p, v, n);
    return hipGetLastError();
}

}  // namespace eclip
