// Implicit-GEMM convolution / linear layer on the gfx950 matrix cores.
//
//   y[m][n] = act( sum_k A[m][k] * w[n][k] + bias[n] + res[m][n] )
//   m = (b, oh, ow)  row of the output in channels-last order
//   k = (kh, kw, ci) with ci innermost, so that 8 consecutive k are 16 contiguous bytes of the
//       input whenever Cin % 8 == 0 (the loader pads the 3-channel network input to 8)
//   A[m][k] = x[b][oh*stride-pad+kh][ow*stride-pad+kw][ci], zero outside the image
//
// A linear layer is the case KH = KW = 1, H = W = 1 (or W = sequence length).
//
// Tiling: one 256-thread workgroup (4 wavefronts of 64) owns a BM x BN output tile and walks K in
// steps of 32 through LDS.  Global loads for step t+1 are issued before the MFMAs of step t.  Each
// wavefront owns a (BM/WM) x (BN/WN) sub-tile made of 16x16 blocks, one v_mfma_f32_16x16x32 per block
// and K step.  The weight tile is fed as the MFMA's row operand and the im2col tile as its column
// operand, so a lane ends up with 4 consecutive output channels of one output pixel, which is 8
// contiguous bytes of y.
//
// Small problems (batch-1 inference: a few dozen tiles) are cut along K into `splits` slices, one
// workgroup each; slices write float partial sums to a workspace, and the workgroup that arrives last
// at the tile's counter adds them in slice order (so the result does not depend on arrival order),
// applies the epilogue and resets the counter.
#include "device_common.h"
#include "kernels.h"

namespace eclip {

namespace {

constexpr int BK = 32;    // K elements per main-loop step
constexpr int LDK = 40;   // LDS row pitch in elements: 80 bytes keeps 16-byte reads of 16 rows conflict-free

struct GemmDev {
    const uint16_t *x, *w, *bias, *res;
    uint16_t *y;
    float *y32;
    float *ws;
    unsigned *counters;
    int B, H, W, Cin, Ho, Wo, KH, KW, stride, pad, act;
    int M, N, K, KT, kt_per, splits, tiles_m;
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
template <typename T>
__device__ __forceinline__ void epilogue_store(const GemmDev &p, int m, int n, f32x4 v)
{
    if (m >= p.M || n >= p.N) return;
    const long off = (long)m * p.N + n;
    float o[4] = {v[0], v[1], v[2], v[3]};
    const bool vec = ((p.N & 3) == 0);      // then n + 3 < N and every access below is aligned
    if (vec) {
        if (p.bias) {
            const uint2 q = *reinterpret_cast<const uint2 *>(p.bias + n);
            o[0] += Cvt<T>::from_bits(q.x & 0xffffu); o[1] += Cvt<T>::from_bits(q.x >> 16);
            o[2] += Cvt<T>::from_bits(q.y & 0xffffu); o[3] += Cvt<T>::from_bits(q.y >> 16);
        }
        if (p.res) {
            const uint2 q = *reinterpret_cast<const uint2 *>(p.res + off);
            o[0] += Cvt<T>::from_bits(q.x & 0xffffu); o[1] += Cvt<T>::from_bits(q.x >> 16);
            o[2] += Cvt<T>::from_bits(q.y & 0xffffu); o[3] += Cvt<T>::from_bits(q.y >> 16);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) o[r] = apply_act(p.act, o[r]);
        if (p.y32) {
            *reinterpret_cast<float4 *>(p.y32 + off) = make_float4(o[0], o[1], o[2], o[3]);
        } else {
            uint2 q;
            q.x = Cvt<T>::to_bits(o[0]) | (Cvt<T>::to_bits(o[1]) << 16);
            q.y = Cvt<T>::to_bits(o[2]) | (Cvt<T>::to_bits(o[3]) << 16);
            *reinterpret_cast<uint2 *>(p.y + off) = q;
        }
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (n + r >= p.N) break;
            float t = o[r];
            if (p.bias) t += Cvt<T>::from_bits(p.bias[n + r]);
            if (p.res) t += Cvt<T>::from_bits(p.res[off + r]);
            t = apply_act(p.act, t);
            if (p.y32) p.y32[off + r] = t;
            else p.y[off + r] = (uint16_t)Cvt<T>::to_bits(t);
        }
    }
}

template <typename T, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(256) void conv_gemm_kernel(GemmDev p)
{
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    constexpr int TM = BM / WM / 16, TN = BN / WN / 16;
    constexpr int A_CH = BM * 4, B_CH = BN * 4;          // 16-byte chunks per K step
    constexpr int A_IT = (A_CH + 255) / 256, B_IT = (B_CH + 255) / 256;

    __shared__ __attribute__((aligned(16))) uint16_t sA[BM * LDK];
    __shared__ __attribute__((aligned(16))) uint16_t sB[BN * LDK];
    __shared__ int s_last;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int tile_m = blockIdx.x % p.tiles_m, tile_n = blockIdx.x / p.tiles_m;
    const int z = blockIdx.y;
    const int m_base = tile_m * BM, n_base = tile_n * BN;

    // ---- per-thread, per-chunk addressing that does not change along K
    bool a_ok[A_IT];
    long a_base[A_IT];
    int a_ih0[A_IT], a_iw0[A_IT];
    const int HoWo = p.Ho * p.Wo;
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
        const int c = tid + it * 256;
        const int m = m_base + (c >> 2);
        a_ok[it] = (c < A_CH) && (m < p.M);
        const int mm = a_ok[it] ? m : 0;
        const int b = mm / HoWo, r = mm - b * HoWo;
        const int oh = r / p.Wo, ow = r - oh * p.Wo;
        a_base[it] = (long)b * p.H * p.W * p.Cin;
        a_ih0[it] = oh * p.stride - p.pad;
        a_iw0[it] = ow * p.stride - p.pad;
    }
    bool b_ok[B_IT];
    long b_base[B_IT];
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
        const int c = tid + it * 256;
        const int n = n_base + (c >> 2);
        b_ok[it] = (c < B_CH) && (n < p.N);
        b_base[it] = (long)(b_ok[it] ? n : 0) * p.K;
    }
    const int kc = (tid & 3) * 8;     // same for every chunk of this thread: 256 % 4 == 0

    uint4 ra[A_IT], rb[B_IT];
    auto load_tile = [&](int kt) {
        const int k = kt * BK + kc;
        const bool k_ok = k < p.K;
        int kh = 0, kw = 0, ci = k;
        if (p.KH * p.KW != 1) {
            const int tap = k / p.Cin;
            ci = k - tap * p.Cin;
            kh = tap / p.KW;
            kw = tap - kh * p.KW;
        }
#pragma unroll
        for (int it = 0; it < A_IT; ++it) {
            uint4 v = make_uint4(0, 0, 0, 0);
            const int ih = a_ih0[it] + kh, iw = a_iw0[it] + kw;
            if (a_ok[it] && k_ok && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W)
                v = *reinterpret_cast<const uint4 *>(p.x + a_base[it] + ((long)ih * p.W + iw) * p.Cin + ci);
            ra[it] = v;
        }
#pragma unroll
        for (int it = 0; it < B_IT; ++it) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (b_ok[it] && k_ok) v = *reinterpret_cast<const uint4 *>(p.w + b_base[it] + k);
            rb[it] = v;
        }
    };

    f32x4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int kt_begin = z * p.kt_per;
    const int kt_end = min(p.KT, kt_begin + p.kt_per);
    const int frag_row = lane & 15, frag_k = (lane >> 4) * 8;

    if (kt_begin < kt_end) load_tile(kt_begin);
    for (int kt = kt_begin; kt < kt_end; ++kt) {
#pragma unroll
        for (int it = 0; it < A_IT; ++it) {
            const int c = tid + it * 256;
            if (c < A_CH) *reinterpret_cast<uint4 *>(&sA[(c >> 2) * LDK + kc]) = ra[it];
        }
#pragma unroll
        for (int it = 0; it < B_IT; ++it) {
            const int c = tid + it * 256;
            if (c < B_CH) *reinterpret_cast<uint4 *>(&sB[(c >> 2) * LDK + kc]) = rb[it];
        }
        __syncthreads();
        if (kt + 1 < kt_end) load_tile(kt + 1);

        uint4 fa[TM], fb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[i] = *reinterpret_cast<const uint4 *>(&sA[(wm * (BM / WM) + i * 16 + frag_row) * LDK + frag_k]);
#pragma unroll
        for (int j = 0; j < TN; ++j)
            fb[j] = *reinterpret_cast<const uint4 *>(&sB[(wn * (BN / WN) + j * 16 + frag_row) * LDK + frag_k]);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = Mma<T>::run(fb[j], fa[i], acc[i][j]);
        __syncthreads();
    }

    // lane owns output pixel m0 + (lane & 15) and channels n0 + 4*(lane >> 4) .. +3 of each 16x16 block
    const int m_l = m_base + wm * (BM / WM) + (lane & 15);
    const int n_l = n_base + wn * (BN / WN) + (lane >> 4) * 4;

    if (p.splits == 1) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) epilogue_store<T>(p, m_l + i * 16, n_l + j * 16, acc[i][j]);
        return;
    }

    // ---- split-K: publish this slice, the last slice to arrive reduces
    const bool vec = ((p.N & 3) == 0);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int m = m_l + i * 16, n = n_l + j * 16;
            if (m >= p.M || n >= p.N) continue;
            float *dst = p.ws + ((long)z * p.M + m) * p.N + n;
            if (vec) {
                *reinterpret_cast<float4 *>(dst) = make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
            } else {
                for (int r = 0; r < 4 && n + r < p.N; ++r) dst[r] = acc[i][j][r];
            }
        }
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const unsigned prev = atomicAdd(&p.counters[blockIdx.x], 1u);
        s_last = (prev == (unsigned)p.splits - 1u);
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int m = m_l + i * 16, n = n_l + j * 16;
            if (m >= p.M || n >= p.N) continue;
            f32x4 s = {0.f, 0.f, 0.f, 0.f};
            for (int zz = 0; zz < p.splits; ++zz) {
                const float *src = p.ws + ((long)zz * p.M + m) * p.N + n;
                if (vec) {
                    const float4 q = *reinterpret_cast<const float4 *>(src);
                    s[0] += q.x; s[1] += q.y; s[2] += q.z; s[3] += q.w;
                } else {
                    for (int r = 0; r < 4 && n + r < p.N; ++r) s[r] += src[r];
                }
            }
            epilogue_store<T>(p, m, n, s);
        }
    if (tid == 0) p.counters[blockIdx.x] = 0u;
}

template <typename T>
hipError_t launch_t(const GemmDev &d, const GemmPlan &pl, hipStream_t s)
{
    const dim3 grid((unsigned)pl.tiles, (unsigned)pl.splits), block(256);
    switch (pl.variant) {
    case 0: hipLaunchKernelGGL((conv_gemm_kernel<T, 128, 128, 2, 2>), grid, block, 0, s, d); break;
    case 1: hipLaunchKernelGGL((conv_gemm_kernel<T, 64, 64, 2, 2>), grid, block, 0, s, d); break;
    default: hipLaunchKernelGGL((conv_gemm_kernel<T, 32, 64, 1, 4>), grid, block, 0, s, d); break;
    }
    return hipGetLastError();
}

}  // namespace

void conv_gemm_tile(int variant, int *bm, int *bn)
{
    static const int t[3][2] = {{128, 128}, {64, 64}, {32, 64}};
    const int v = variant < 0 ? 0 : (variant > 2 ? 2 : variant);
    *bm = t[v][0];
    *bn = t[v][1];
}

static long cdiv(long a, long b) { return (a + b - 1) / b; }

GemmPlan conv_gemm_plan(long M, long N, long K, int n_cu, size_t ws_floats, size_t n_counters)
{
    const long KT = cdiv(K, BK);
    auto tiles = [&](int v) { int bm, bn; conv_gemm_tile(v, &bm, &bn); return cdiv(M, bm) * cdiv(N, bn); };
    GemmPlan pl{1, 1, 0};
    if (tiles(0) >= 2L * n_cu) pl.variant = 0;
    else if (tiles(1) >= n_cu) pl.variant = 1;
    else pl.variant = (tiles(1) * 2 <= n_cu || M <= 32) ? 2 : 1;
    pl.tiles = (int)tiles(pl.variant);
    if (pl.tiles < n_cu && KT >= 8 && (size_t)pl.tiles <= n_counters) {
        long want = cdiv(n_cu, pl.tiles);
        long cap = KT / 4;                       // at least 4 K steps per slice
        long s = want < cap ? want : cap;
        if (s > 32) s = 32;
        while (s > 1 && (size_t)(s * M * N) > ws_floats) --s;
        if (s > 1) {
            const long kt_per = cdiv(KT, s);
            pl.splits = (int)cdiv(KT, kt_per);
        }
    }
    return pl;
}

hipError_t launch_conv_gemm(const ConvGemmArgs &a, const GemmPlan &pl, hipStream_t s)
{
    GemmDev d;
    d.x = (const uint16_t *)a.x; d.w = (const uint16_t *)a.w; d.bias = (const uint16_t *)a.bias;
    d.res = (const uint16_t *)a.res; d.y = (uint16_t *)a.y; d.y32 = a.y32; d.ws = a.ws; d.counters = a.counters;
    d.B = a.B; d.H = a.H; d.W = a.W; d.Cin = a.Cin; d.Ho = a.Ho; d.Wo = a.Wo; d.KH = a.KH; d.KW = a.KW;
    d.stride = a.stride; d.pad = a.pad; d.act = a.act;
    d.M = a.B * a.Ho * a.Wo; d.N = a.Cout; d.K = a.KH * a.KW * a.Cin;
    d.KT = (d.K + BK - 1) / BK;
    d.splits = pl.splits;
    d.kt_per = (d.KT + pl.splits - 1) / pl.splits;
    int bm, bn;
    conv_gemm_tile(pl.variant, &bm, &bn);
    d.tiles_m = (d.M + bm - 1) / bm;
    if (a.dtype == DT_BF16) return launch_t<bf16_t>(d, pl, s);
    return launch_t<f16_t>(d, pl, s);
}

}  // namespace eclip
