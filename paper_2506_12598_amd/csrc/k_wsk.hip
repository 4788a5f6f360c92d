// Wave-split-K implicit GEMM for the small, latency-bound layers of batch-1 inference.
//
// Same contraction as the LDS-tiled kernel (y[m][n] = act(sum_k A[m][k] w[n][k] + bias + res)), but the
// parallelism is taken from K *inside* the workgroup instead of from a second kernel:
//   - a workgroup of NW wavefronts owns one (TM*16) x (TN*16) output tile;
//   - wavefront w multiplies the whole tile over its own contiguous slice of K, reading its MFMA
//     operands straight from global memory (each lane 16 bytes = 8 consecutive k of one row), several K
//     steps in flight, with no LDS staging and no barrier in the loop: every element of the A and W
//     tiles is still read exactly once per workgroup, because the slices are disjoint;
//   - the NW partial tiles meet in LDS (float, lane-contiguous so the writes are conflict-free), and
//     after one barrier the first TM*TN*64 threads add them in wavefront order and apply the epilogue.
// With a few dozen tiles per layer this fills the machine with NW x tiles wavefronts without the
// workspace round trip and second launch of a grid-level K split, and the summation order is fixed.
#include "gemm_common.h"
#include "kernels.h"

namespace eclip {

namespace {

// Sum of the NW wavefronts' partial tiles (in LDS, block (i, j) of wavefront w at red4[(w * TM * TN + i * TN + j) * 64 + lane])
// with bias, residual and the activation ACT, written to the output.
template <typename T, int TM, int TN, int NW, int ACT>
__device__ __forceinline__ void wsk_finish(const GemmDev &p, const float4 *red4, int m_base, int n_base)
{
    constexpr int BM = TM * 16, BN = TN * 16;
    const int tid = threadIdx.x;
    if ((p.N & 7) == 0 && p.M * p.N >= (1 << 20)) {
        // large outputs: one thread per (row, 8 consecutive channels): its two float4 of every partial tile sit 16
        // lanes apart; stores are 16 bytes per lane along the rows instead of 8 bytes to each of 16 rows.  (Small
        // outputs keep the form below: twice the threads share the summation, which matters more there.)
        constexpr int C8 = BN / 8;
        for (int t = tid; t < BM * C8; t += NW * 64) {
            const int r = t / C8, c8 = t - r * C8;
            const int blk = (r >> 4) * TN + (c8 >> 1), l0 = (c8 & 1) * 32 + (r & 15);
            f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const float4 q0 = red4[(w * (TM * TN) + blk) * 64 + l0], q1 = red4[(w * (TM * TN) + blk) * 64 + l0 + 16];
                s0[0] += q0.x; s0[1] += q0.y; s0[2] += q0.z; s0[3] += q0.w;
                s1[0] += q1.x; s1[1] += q1.y; s1[2] += q1.z; s1[3] += q1.w;
            }
            const int m = m_base + r, n = n_base + c8 * 8;
            if (m < p.M && n < p.N) {
                float o[8] = {s0[0], s0[1], s0[2], s0[3], s1[0], s1[1], s1[2], s1[3]};
                epilogue_store8<T, ACT>(p.bias, p.res, p.y, p.y32, p.ldy, m, n, o);
            }
        }
        return;
    }
    for (int slot = tid; slot < TM * TN * 64; slot += NW * 64) {
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float4 q = red4[w * (TM * TN * 64) + slot];
            s[0] += q.x; s[1] += q.y; s[2] += q.z; s[3] += q.w;
        }
        const int blk = slot >> 6, l = slot & 63;
        const int i = blk / TN, j = blk - i * TN;
        // lane l of block (i, j) holds output pixel 16*i + (l & 15), channels 16*j + 4*(l >> 4) .. +3
        epilogue_store<T, ACT>(p.bias, p.res, p.y, p.y32, p.M, p.N, m_base + i * 16 + (l & 15), n_base + j * 16 + (l >> 4) * 4, s, 4, p.ldy);
    }
}

// NCHW: the first layer of an image model reads the caller's [B][C][H][W] tensor (C = p.nchw_c <= 4) directly.  Its
// K runs over (kh, kw, 8 channel slots), one 16-byte chunk per tap as in the channels-last copy with C padded to 8, so
// weights and bookkeeping are the same; the chunk is put together from C two-byte loads, one per plane.
template <typename T, int TM, int TN, int NW, int D, bool NCHW = false>
__global__ __launch_bounds__(NW * 64) void conv_wsk_kernel(GemmDev p0, GemmDev p1, int n0)
{
    // One launch can carry two independent layers ("horizontal" fusion, e.g. the two convolutions that read a
    // residual block's input): workgroups 0 .. n0-1 work on p0, the rest on p1.  A single layer passes n0 = grid.
    const bool second = (int)blockIdx.x >= n0;
    const GemmDev &p = second ? p1 : p0;
    const int bid = (int)blockIdx.x - (second ? n0 : 0);
    extern __shared__ __attribute__((aligned(16))) float red[];    // [NW][TM*TN][64][4]
    constexpr int BM = TM * 16, BN = TN * 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Workgroup b runs on XCD b % 8, and each XCD has its own L2.  With raster 2 (3) the tiles are dealt so that an
    // XCD owns a contiguous range of tile columns (rows): the larger operand, the weights (the activations), is then
    // fetched from memory by one XCD only instead of by all eight.
    int tile_m, tile_n;
    if (p.raster == 2) {
        const int xcd = bid & 7, q = bid >> 3, per = (p.tiles_n + 7) >> 3, r = q / p.tiles_m;
        tile_m = q - r * p.tiles_m;
        tile_n = xcd * per + r;
        if (r >= per || tile_n >= p.tiles_n) return;
    } else if (p.raster == 3) {
        const int xcd = bid & 7, q = bid >> 3, per = (p.tiles_m + 7) >> 3, r = q / p.tiles_n;
        tile_n = q - r * p.tiles_n;
        tile_m = xcd * per + r;
        if (r >= per || tile_m >= p.tiles_m) return;
    } else {
        tile_m = bid % p.tiles_m;
        tile_n = bid / p.tiles_m;
    }
    const int m_base = tile_m * BM, n_base = tile_n * BN;
    // The im2col operand is loaded in "tile order": lane l takes row l >> 2, 16-byte chunk l & 3 of the step's 64 bytes, so
    // that four neighbouring lanes read one 64-byte run (measured per CU, L2-resident: 65 GB/s, against 36 GB/s when
    // lane l reads row l & 15, chunk l >> 4 as the matrix instruction wants its operand).  Before it is used the
    // fragment is moved into that order across the lanes, four ds_bpermute (the LDS crossbar, no LDS memory).
    const int row = lane >> 2, g = lane & 3;
    const int perm_src = (((lane & 15) << 2) | (lane >> 4)) << 2;      // byte address of the lane that holds this lane's chunk

    // rows of the im2col operand (one per 16x16 block row) and of the weight operand
    // buffer descriptors: lanes without a valid chunk use an offset past the end and receive zeros
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, (int)p.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void *)p.w, 0, (int)p.w_bytes, 0x00020000);
    constexpr unsigned OOB = 0xffffffffu;
    int a_ok[TM];
    unsigned a_off0[TM];                     // byte offset of pixel (ih0, iw0) of the row's image (modulo 2^32 when padded)
    int a_ih0[TM], a_iw0[TM];
    const int HoWo = p.Ho * p.Wo;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m_base + i * 16 + row;
        a_ok[i] = m < p.M;
        const int mm = a_ok[i] ? m : 0;
        const int b = mm / HoWo, r = mm - b * HoWo;
        const int oh = r / p.Wo, ow = r - oh * p.Wo;
        a_ih0[i] = oh * p.stride - p.pad;
        a_iw0[i] = ow * p.stride - p.pad;
        if constexpr (NCHW) a_off0[i] = ((unsigned)(b * p.nchw_c) * (unsigned)(p.H * p.W) + (unsigned)(a_ih0[i] * p.W + a_iw0[i])) * 2u;
        else a_off0[i] = ((unsigned)b * (unsigned)(p.H * p.W) + (unsigned)(a_ih0[i] * p.W + a_iw0[i])) * (unsigned)p.ldx * 2u;
    }
    const unsigned plane = (unsigned)(p.H * p.W) * 2u;            // NCHW: bytes between the planes of two channels
    // weights: 1 KB blocks of 16 rows x 32 k in lane order, so a fragment is one contiguous load
    const int KB = (p.K + 31) >> 5, NB = (p.N + 15) >> 4;
    int b_ok[TN];
    unsigned b_base[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int nb = (n_base >> 4) + j;
        b_ok[j] = nb < NB;
        b_base[j] = ((unsigned)(b_ok[j] ? nb : 0) * (unsigned)KB * 64u + (unsigned)lane) * 16u;
    }

    // this wavefront's K steps (32 k each)
    const int ksteps = (p.K + 31) / 32;
    const int per_wave = (ksteps + NW - 1) / NW;
    const int ks0 = min(ksteps, wave * per_wave), ks1 = min(ksteps, ks0 + per_wave);
    const int n_steps = ks1 - ks0;
    const int k_lim = min(p.K, ks1 * 32);

    // running position of this lane's next 8 k: k = (kh, kw, ci), advanced by 32 per step without dividing
    int k = ks0 * 32 + g * 8, kb = ks0;
    int kh = 0, kw = 0, ci = k;
    if (p.KH * p.KW != 1) {
        const int tap = k / p.Cin;
        ci = k - tap * p.Cin;
        kh = tap / p.KW;
        kw = tap - kh * p.KW;
    }
    struct Frag { uint4 a[TM]; uint4 b[TN]; };
    // branch-free: a lane whose chunk is padding, beyond M / N or beyond the wavefront's K slice loads zeros
    auto load = [&](Frag &f) {
        const int k_ok = k < k_lim, kb_ok = kb < ks1;
        const unsigned tap_off = NCHW ? (unsigned)(kh * p.W + kw) * 2u : (unsigned)((kh * p.W + kw) * p.ldx + ci) * 2u;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int ok = a_ok[i] & k_ok & (int)((unsigned)(a_ih0[i] + kh) < (unsigned)p.H) & (int)((unsigned)(a_iw0[i] + kw) < (unsigned)p.W);
            if constexpr (NCHW) {
                unsigned c[4];
#pragma unroll
                for (int ch = 0; ch < 3; ++ch)
                    c[ch] = (unsigned)__builtin_amdgcn_raw_buffer_load_b16(rx, (ok & (int)(ch < p.nchw_c)) ? a_off0[i] + tap_off + (unsigned)ch * plane : OOB, 0, 0) & 0xffffu;
                c[3] = 0u;
                if (p.nchw_c > 3)                      // uniform; RGB inputs skip the fourth load
                    c[3] = (unsigned)__builtin_amdgcn_raw_buffer_load_b16(rx, ok ? a_off0[i] + tap_off + 3u * plane : OOB, 0, 0) & 0xffffu;
                f.a[i] = make_uint4(c[0] | (c[1] << 16), c[2] | (c[3] << 16), 0u, 0u);
            } else {
                const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? a_off0[i] + tap_off : OOB, 0, 0);
                f.a[i] = make_uint4(v.x, v.y, v.z, v.w);
            }
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rw, (b_ok[j] & kb_ok) ? b_base[j] + (unsigned)kb * 1024u : OOB, 0, 0);
            f.b[j] = make_uint4(v.x, v.y, v.z, v.w);
        }
        k += 32;
        ++kb;
        ci += 32;
        // Cin >= 8, so 4 turns always suffice; for a 1x1 window Cin == K and a wrap only happens beyond K
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int wrap = ci >= p.Cin;
            ci -= wrap ? p.Cin : 0;
            kw += wrap;
            const int wrap2 = kw == p.KW;
            kw = wrap2 ? 0 : kw;
            kh += wrap2;
        }
    };

    f32x4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    // moves the im2col fragments of one step into the lane order of the matrix instruction
    auto permute = [&](const Frag &f, uint4 (&a)[TM]) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            a[i].x = (unsigned)__builtin_amdgcn_ds_bpermute(perm_src, (int)f.a[i].x);
            a[i].y = (unsigned)__builtin_amdgcn_ds_bpermute(perm_src, (int)f.a[i].y);
            a[i].z = (unsigned)__builtin_amdgcn_ds_bpermute(perm_src, (int)f.a[i].z);
            a[i].w = (unsigned)__builtin_amdgcn_ds_bpermute(perm_src, (int)f.a[i].w);
        }
    };

    // D steps of loads in flight per wavefront (the fewer registers a step takes, the deeper); a short slice is
    // loaded whole before the first matrix instruction.  Steps beyond the slice load zeros and add nothing.  The
    // lane exchange of step d + 1 is issued before the matrix instructions of step d, which hide its latency (after
    // the last step it moves stale data that nothing reads).
    Frag f[D];
    static_for<D>([&](auto dc) { load(f[decltype(dc)::value]); });
    uint4 pa[TM];
    permute(f[0], pa);
    for (int s = 0; s < n_steps; s += D) {
        const bool more = s + D < n_steps;       // wavefront-uniform
        static_for<D>([&](auto dc) {
            constexpr int d = decltype(dc)::value;
            uint4 pn[TM];
            permute(f[(d + 1) % D], pn);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = Mma<T>::run(f[d].b[j], pa[i], acc[i][j]);
            if (more) load(f[d]);
#pragma unroll
            for (int i = 0; i < TM; ++i) pa[i] = pn[i];
        });
    }

    // ---- cross-wavefront sum through LDS
    float4 *red4 = reinterpret_cast<float4 *>(red);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
            red4[(wave * (TM * TN) + i * TN + j) * 64 + lane] = make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
    __syncthreads();
#define FIN(A) wsk_finish<T, TM, TN, NW, A>(p, red4, m_base, n_base)
    ECLIP_ACT_SWITCH(p.act, FIN)
#undef FIN
}

// prefetch depth per tile shape: about 24 / (TM + TN) steps of 16-byte loads per lane
// (16 wavefronts leave 128 registers per lane, which holds only two steps of a 32x64 tile)
template <int TM, int TN, int NW> struct Depth {
    static constexpr int value = (TM + TN) <= 2 ? 8 : (TM + TN) <= 3 ? 6 : (TM + TN) <= 5 ? (NW == 16 ? 3 : 4) : (TM + TN) <= 6 ? (NW == 16 ? 2 : 3) : 2;
};

template <typename T, int TM, int TN>
hipError_t launch_nw(const GemmDev &d, const GemmDev &d1, int n0, int nw, int tiles, hipStream_t s)
{
    const size_t lds = (size_t)nw * TM * TN * 64 * 16;
    if (lds > 128 * 1024) return hipErrorInvalidValue;
    const dim3 grid((unsigned)tiles);
    if (d.nchw_c) {                                    // first-layer form: 4 wavefronts, tiles 16x64, 32x64, 32x32
        if constexpr ((TM == 1 && TN == 4) || (TM == 2 && TN == 4) || (TM == 2 && TN == 2)) {
            if (nw != 4 || &d != &d1) return hipErrorInvalidValue;
            hipLaunchKernelGGL((conv_wsk_kernel<T, TM, TN, 4, Depth<TM, TN, 4>::value, true>), grid, dim3(256), lds, s, d, d1, n0);
            return hipGetLastError();
        } else {
            return hipErrorInvalidValue;
        }
    }
    switch (nw) {
    case 4: hipLaunchKernelGGL((conv_wsk_kernel<T, TM, TN, 4, Depth<TM, TN, 4>::value>), grid, dim3(256), lds, s, d, d1, n0); break;
    case 8: hipLaunchKernelGGL((conv_wsk_kernel<T, TM, TN, 8, Depth<TM, TN, 8>::value>), grid, dim3(512), lds, s, d, d1, n0); break;
    case 16:
        if constexpr (TM * TN <= 8) hipLaunchKernelGGL((conv_wsk_kernel<T, TM, TN, 16, Depth<TM, TN, 16>::value>), grid, dim3(1024), lds, s, d, d1, n0);
        else return hipErrorInvalidValue;        // 16 partial 64x64 tiles would not fit in LDS
        break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <typename T>
hipError_t launch_tile(const GemmDev &d, const GemmDev &d1, int n0, int variant, int nw, int tiles, hipStream_t s)
{
    switch (variant) {
    case 0: return launch_nw<T, 1, 4>(d, d1, n0, nw, tiles, s);
    case 1: return launch_nw<T, 2, 4>(d, d1, n0, nw, tiles, s);
    case 2: return launch_nw<T, 4, 4>(d, d1, n0, nw, tiles, s);
    case 3: return launch_nw<T, 1, 1>(d, d1, n0, nw, tiles, s);
    case 4: return launch_nw<T, 1, 2>(d, d1, n0, nw, tiles, s);
    case 5: return launch_nw<T, 2, 2>(d, d1, n0, nw, tiles, s);
    default: return hipErrorInvalidValue;
    }
}

template <typename T, int TM, int TN>
hipError_t set_attr_tile()
{
    hipError_t e;
    const int lim = 144 * 1024;
    if ((e = hipFuncSetAttribute((const void *)conv_wsk_kernel<T, TM, TN, 4, Depth<TM, TN, 4>::value>, hipFuncAttributeMaxDynamicSharedMemorySize, lim)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute((const void *)conv_wsk_kernel<T, TM, TN, 8, Depth<TM, TN, 8>::value>, hipFuncAttributeMaxDynamicSharedMemorySize, lim)) != hipSuccess) return e;
    if constexpr (TM * TN <= 8)
        return hipFuncSetAttribute((const void *)conv_wsk_kernel<T, TM, TN, 16, Depth<TM, TN, 16>::value>, hipFuncAttributeMaxDynamicSharedMemorySize, lim);
    return hipSuccess;
}

}  // namespace

void conv_wsk_tile(int variant, int *bm, int *bn)
{
    static const int t[CONV_WSK_VARIANTS][2] = {{16, 64}, {32, 64}, {64, 64}, {16, 16}, {16, 32}, {32, 32}};
    const int v = variant < 0 ? 0 : (variant >= CONV_WSK_VARIANTS ? CONV_WSK_VARIANTS - 1 : variant);
    *bm = t[v][0];
    *bn = t[v][1];
}

size_t conv_wsk_lds_bytes(int variant, int nw)
{
    int bm, bn;
    conv_wsk_tile(variant, &bm, &bn);
    return (size_t)nw * bm * bn * 4;
}

hipError_t conv_wsk_init()
{
    hipError_t e;
#define SET(T)                                                     \
    if ((e = set_attr_tile<T, 1, 4>()) != hipSuccess) return e;    \
    if ((e = set_attr_tile<T, 2, 4>()) != hipSuccess) return e;    \
    if ((e = set_attr_tile<T, 4, 4>()) != hipSuccess) return e;    \
    if ((e = set_attr_tile<T, 1, 1>()) != hipSuccess) return e;    \
    if ((e = set_attr_tile<T, 1, 2>()) != hipSuccess) return e;    \
    if ((e = set_attr_tile<T, 2, 2>()) != hipSuccess) return e;
    SET(bf16_t)
    SET(f16_t)
#undef SET
    return hipSuccess;
}

hipError_t launch_conv_wsk(const GemmDev &d, int dtype, int variant, int nw, int tiles, hipStream_t s)
{
    if (dtype == DT_BF16) return launch_tile<bf16_t>(d, d, tiles, variant, nw, tiles, s);
    return launch_tile<f16_t>(d, d, tiles, variant, nw, tiles, s);
}

hipError_t launch_conv_wsk_pair(const GemmDev &d0, int tiles0, const GemmDev &d1, int tiles1, int dtype, int variant, int nw, hipStream_t s)
{
    if (dtype == DT_BF16) return launch_tile<bf16_t>(d0, d1, tiles0, variant, nw, tiles0 + tiles1, s);
    return launch_tile<f16_t>(d0, d1, tiles0, variant, nw, tiles0 + tiles1, s);
}

}  // namespace eclip
