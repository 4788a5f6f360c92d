// Grouped convolution (1 < groups < channels) on the matrix cores.
//
// A grouped convolution is a dense one whose weight matrix is block-diagonal.  Groups of a few channels are far
// narrower than the 32-deep, 16-wide operands of the matrix instruction, so S neighbouring groups are taken together
// as one "super-group": its S*cig input channels and S*cog output channels form a small dense problem whose weight
// block holds the S group blocks on its diagonal and zeros elsewhere (S is the smallest divisor of `groups` that makes
// S*cig a multiple of 32 and S*cog a multiple of 16, see gconv_mfma_pick).  The zeros are multiplied like any other
// value — with S = 8 seven eighths of the multiply-adds are wasted — which is still far cheaper than the scalar
// multiply-adds of the direct kernel: a ResNeXt 3x3 layer at 56x56 is 29 MFLOP of real work.
//
// Work split: a wavefront owns TM blocks of 16 output pixels x NBC blocks of 16 output channels of one super-group and
// runs over all of K = taps x S*cig alone; there is no LDS and no barrier.  Its operands come straight from memory,
// D steps of 32 k ahead: the activation chunk in tile order (lane l: pixel l >> 2, 16-byte chunk l & 3, so that four
// neighbouring lanes read one 64-byte run) and moved to the order the matrix instruction wants across the lanes with
// ds_bpermute; the weights from 1 KB blocks already stored in that order (block (sg, nb, t) at
// ((sg * NB + nb) * KT + t) KB, t = tap * (S*cig / 32) + kb).  The four wavefronts of a workgroup take neighbouring
// pixel blocks of the same super-group, so they share its weights in the L1.
#include "gemm_common.h"
#include "kernels.h"

namespace eclip {

namespace {

struct GConvDev {
    const uint16_t *x, *w, *bias, *res;
    uint16_t *y;
    int B, H, W, Cin, Ho, Wo, Cout, KH, KW, stride, pad, act;
    int M, SI, SO, n_sg, n_chunks, m_tiles;
    unsigned x_bytes, w_bytes;
};

template <typename T, int TM, int NBC, int D>
__global__ __launch_bounds__(256) void gconv_mfma_kernel(GConvDev p)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tile_m = (int)blockIdx.x % p.m_tiles, unit = (int)blockIdx.x / p.m_tiles;
    const int sg = unit / p.n_chunks, nc = unit - sg * p.n_chunks;
    const int m_base = (tile_m * 4 + wave) * (TM * 16);
    if (m_base >= p.M) return;                                   // no barrier below: a whole wavefront may leave
    const int row = lane >> 2, g = lane & 3;
    const int perm_src = (((lane & 15) << 2) | (lane >> 4)) << 2;

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, (int)p.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void *)p.w, 0, (int)p.w_bytes, 0x00020000);
    constexpr unsigned OOB = 0xffffffffu;
    int a_ok[TM], a_ih0[TM], a_iw0[TM];
    unsigned a_off0[TM];
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
        a_off0[i] = (((unsigned)b * (unsigned)(p.H * p.W) + (unsigned)(a_ih0[i] * p.W + a_iw0[i])) * (unsigned)p.Cin + (unsigned)(sg * p.SI + g * 8)) * 2u;
    }
    const int KBS = p.SI >> 5, KT = p.KH * p.KW * KBS, NB = p.SO >> 4;
    int b_ok[NBC];
    unsigned b_base[NBC];
#pragma unroll
    for (int j = 0; j < NBC; ++j) {
        const int nb = nc * NBC + j;
        b_ok[j] = nb < NB;
        b_base[j] = ((unsigned)((sg * NB + (b_ok[j] ? nb : 0)) * KT) * 64u + (unsigned)lane) * 16u;
    }

    // running position of the next step to load: tap (kh, kw), 32-channel block kb of the super-group
    int t = 0, kh = 0, kw = 0, kb = 0;
    struct Frag { uint4 a[TM]; uint4 b[NBC]; };
    auto load = [&](Frag &f) {
        const int t_ok = t < KT;
        const unsigned tap_off = (unsigned)((kh * p.W + kw) * p.Cin + kb * 32) * 2u;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int ok = a_ok[i] & t_ok & (int)((unsigned)(a_ih0[i] + kh) < (unsigned)p.H) & (int)((unsigned)(a_iw0[i] + kw) < (unsigned)p.W);
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? a_off0[i] + tap_off : OOB, 0, 0);
            f.a[i] = make_uint4(v.x, v.y, v.z, v.w);
        }
#pragma unroll
        for (int j = 0; j < NBC; ++j) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rw, (b_ok[j] & t_ok) ? b_base[j] + (unsigned)t * 1024u : OOB, 0, 0);
            f.b[j] = make_uint4(v.x, v.y, v.z, v.w);
        }
        ++t;
        ++kb;
        const int wrap = kb == KBS;
        kb = wrap ? 0 : kb;
        kw += wrap;
        const int wrap2 = kw == p.KW;
        kw = wrap2 ? 0 : kw;
        kh += wrap2;
    };
    auto permute = [&](const Frag &f, uint4 (&a)[TM]) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            a[i].x = (unsigned)__builtin_amdgcn_ds_bpermute(perm_src, (int)f.a[i].x);
            a[i].y = (unsigned)__builtin_amdgcn_ds_bpermute(perm_src, (int)f.a[i].y);
            a[i].z = (unsigned)__builtin_amdgcn_ds_bpermute(perm_src, (int)f.a[i].z);
            a[i].w = (unsigned)__builtin_amdgcn_ds_bpermute(perm_src, (int)f.a[i].w);
        }
    };

    f32x4 acc[TM][NBC];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < NBC; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // D steps in flight; steps beyond KT load zeros and add nothing
    Frag f[D];
    static_for<D>([&](auto dc) { load(f[decltype(dc)::value]); });
    uint4 pa[TM];
    permute(f[0], pa);
    for (int s = 0; s < KT; s += D) {
        const bool more = s + D < KT;            // wavefront-uniform
        static_for<D>([&](auto dc) {
            constexpr int d = decltype(dc)::value;
            uint4 pn[TM];
            permute(f[(d + 1) % D], pn);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < NBC; ++j) acc[i][j] = Mma<T>::run(f[d].b[j], pa[i], acc[i][j]);
            if (more) load(f[d]);
#pragma unroll
            for (int i = 0; i < TM; ++i) pa[i] = pn[i];
        });
    }

    // lane l of block (i, j) holds output pixel 16*i + (l & 15), channels 16*j + 4*(l >> 4) .. +3 of the chunk
    const int n0 = sg * p.SO + nc * NBC * 16;
#define FIN(A)                                                                                                        \
    _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                                    \
        _Pragma("unroll") for (int j = 0; j < NBC; ++j)                                                               \
            if (b_ok[j])                                                                                              \
                epilogue_store<T, A>(p.bias, p.res, p.y, nullptr, p.M, p.Cout, m_base + i * 16 + (lane & 15),         \
                                     n0 + j * 16 + 4 * (lane >> 4), acc[i][j]);
    ECLIP_ACT_SWITCH(p.act, FIN)
#undef FIN
}

}  // namespace

bool gconv_mfma_pick(int groups, int cig, int cog, int *S_out)
{
    for (int S = 1; S <= groups; ++S) {
        if (groups % S) continue;
        if ((S * cig) % 32 == 0 && (S * cog) % 16 == 0) {
            if (S > 16) return false;            // more than 15/16 of the multiply-adds wasted: the direct kernel
            *S_out = S;
            return true;
        }
    }
    return false;
}

long gconv_mfma_workgroups(long M, int groups, int cog, int S, int n_cu)
{
    const int NB = S * cog / 16, nbc = NB <= 2 ? 2 : 4;
    const long units = (long)(groups / S) * ((NB + nbc - 1) / nbc);
    const long wg1 = (M + 63) / 64 * units;
    return wg1 >= 16L * n_cu ? (M + 127) / 128 * units : wg1;
}

hipError_t launch_gconv_mfma(const GConvArgs &a, int S, int n_cu, hipStream_t s)
{
    const int cig = a.Cin / a.groups, cog = a.Cout / a.groups;
    GConvDev p;
    p.x = (const uint16_t *)a.x; p.w = (const uint16_t *)a.w; p.bias = (const uint16_t *)a.bias; p.res = (const uint16_t *)a.res;
    p.y = (uint16_t *)a.y;
    p.B = a.B; p.H = a.H; p.W = a.W; p.Cin = a.Cin; p.Ho = a.Ho; p.Wo = a.Wo; p.Cout = a.Cout; p.KH = a.KH; p.KW = a.KW;
    p.stride = a.stride; p.pad = a.pad; p.act = a.act;
    const long M = (long)a.B * a.Ho * a.Wo;
    const long xb = (long)a.B * a.H * a.W * a.Cin * 2;
    if (S < 1 || a.groups % S || (S * cig) % 32 || (S * cog) % 16 || a.Cin % 8) return hipErrorInvalidValue;
    p.SI = S * cig; p.SO = S * cog; p.n_sg = a.groups / S;
    const long wb = (long)p.n_sg * (p.SO / 16) * a.KH * a.KW * (p.SI / 32) * 1024;
    if (M >= (1L << 30) || xb >= (1L << 32) - 16 || wb >= (1L << 32) - 16) return hipErrorInvalidValue;
    p.M = (int)M; p.x_bytes = (unsigned)xb; p.w_bytes = (unsigned)wb;
    const int NB = p.SO / 16, kt = a.KH * a.KW * (p.SI / 32);
    const int nbc = NB <= 2 ? 2 : 4;
    p.n_chunks = (NB + nbc - 1) / nbc;
    // One pixel block per wavefront: measured faster than two at every ResNeXt shape up to batch 8 (12.3 against 13.9 us
    // at 25088 x 128, 4.9 against 6.5 us at 392 x 1024: the wavefront's serial chain of loads, lane exchange and stores is
    // what costs, and more wavefronts hide it better than longer ones); two only for grids beyond 16 workgroups per CU.
    const long wg1 = (M + 63) / 64 * p.n_sg * p.n_chunks;
    const int tm = wg1 >= 16L * n_cu ? 2 : 1;
    p.m_tiles = (int)((M + 64 * tm - 1) / (64 * tm));
    const long grid = (long)p.m_tiles * p.n_sg * p.n_chunks;
    if (grid >= (1L << 31)) return hipErrorInvalidValue;
#define GO(T, TM_, NBC_, D_) hipLaunchKernelGGL((gconv_mfma_kernel<T, TM_, NBC_, D_>), dim3((unsigned)grid), dim3(256), 0, s, p)
#define SHAPES(T)                                  \
    if (tm == 1 && nbc == 2 && kt > 8 && kt <= 10) GO(T, 1, 2, 10);   /* a 3 x 3 window over 32 channels: one round of loads */ \
    else if (tm == 1 && nbc == 2) GO(T, 1, 2, 8);  \
    else if (tm == 1) GO(T, 1, 4, 4);              \
    else if (nbc == 2 && kt > 6 && kt <= 10) GO(T, 2, 2, 10); \
    else if (nbc == 2) GO(T, 2, 2, 6);             \
    else GO(T, 2, 4, 4);
    if (a.dtype == DT_BF16) { SHAPES(bf16_t) } else if (a.dtype == DT_F16) { SHAPES(f16_t) } else return hipErrorInvalidValue;
#undef SHAPES
#undef GO
    return hipGetLastError();
}

}  // namespace eclip
