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
// steps of BK through a two-slot LDS ring.  Global loads run two steps ahead of the MFMAs: while step t
// is multiplied out of LDS slot t%2, the registers already hold step t+1 and the loads of step t+2 are
// in flight, so one barrier per step suffices and a load has two steps to arrive.  Each wavefront owns
// a (BM/WM) x (BN/WN) sub-tile made of 16x16 blocks, one v_mfma_f32_16x16x32 per block and 32 k.  The
// weight tile is fed as the MFMA's row operand and the im2col tile as its column operand, so a lane
// ends up with 4 consecutive output channels of one output pixel: 8 contiguous bytes of y.
//
// Batch-1 inference leaves most layers with a few dozen tiles and a long K.  Those are cut along K
// into `splits` slices, one workgroup each, which write float partial sums to a workspace; a second,
// tiny kernel adds the slices in slice order (the sum does not depend on scheduling) and applies the
// epilogue.  The kernel boundary is what makes the partial sums visible: a device-wide fence inside the
// GEMM would have to write back the whole L2 of the issuing XCD, which costs far more than a launch.
#include <cstdio>
#include <cstdlib>

#include "gemm_common.h"
#include "kernels.h"

namespace eclip {

namespace {

template <typename T, int BM, int BN, int BK, int WM, int WN, int RS, bool OVERLAP = false>
__global__ __launch_bounds__(WM * WN * 64) void conv_gemm_kernel(GemmDev p)
{
    constexpr int NT = WM * WN * 64;         // threads per workgroup: 4 wavefronts, 8 for the 256x256 tile
    static_assert(RS % 2 == 0, "register stages alternate between the two LDS slots");
    constexpr int LDK = BK + 8;              // row pitch: 16-byte reads of 16 consecutive rows hit distinct banks
    constexpr int CPR = BK / 8;              // 16-byte chunks per row
    constexpr int TM = BM / WM / 16, TN = BN / WN / 16;
    constexpr int A_CH = BM * CPR, B_CH = BN * CPR;
    constexpr int A_IT = (A_CH + NT - 1) / NT, B_IT = (B_CH + NT - 1) / NT;
    static_assert(NT % CPR == 0, "a thread keeps the same k chunk for all of its rows");

    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];     // sA[2][BM*LDK] then sB[2][BN*LDK]
    uint16_t *const sA0 = smem, *const sB0 = smem + 2 * BM * LDK;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    // Workgroups are handed to the 8 XCDs round-robin (workgroup b runs on XCD b % 8), each XCD has its own
    // L2, and the 32 CUs of an XCD run 32 consecutive workgroups of that XCD at a time.  With `raster` set
    // (large problems) those 32 workgroups form an 8 x 4 block of tiles, so that one K step pulls 8 + 4
    // operand tiles into the L2 instead of up to 32 + 1; blocks are dealt to the XCDs in row-major order.
    int tile_m, tile_n;
    if (p.raster) {
        const int b = blockIdx.x, l = b >> 3, w = l & 31;
        const int sb = (l >> 5) * 8 + (b & 7);
        const int sbm = (p.tiles_m + 7) >> 3;
        tile_m = (sb % sbm) * 8 + (w & 7);
        tile_n = (sb / sbm) * 4 + (w >> 3);
        if (tile_m >= p.tiles_m || tile_n >= p.tiles_n) return;
    } else {
        tile_m = blockIdx.x % p.tiles_m;
        tile_n = blockIdx.x / p.tiles_m;
    }
    const int z = blockIdx.y;
    const int m_base = tile_m * BM, n_base = tile_n * BN;

    // ---- per-thread, per-chunk addressing that does not change along K
    // Operands are read through buffer descriptors: a lane whose chunk is padding, beyond M / N or beyond K
    // is given an offset past the end of the buffer, for which the hardware returns zeros.  This keeps the
    // loads free of branches, so the loads of different K steps are counted apart by the hardware.
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, (int)p.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void *)p.w, 0, (int)p.w_bytes, 0x00020000);
    constexpr unsigned OOB = 0xffffffffu;
    bool a_ok[A_IT];
    unsigned a_base[A_IT];                   // byte offset of the image the row belongs to
    int a_ih0[A_IT], a_iw0[A_IT];
    const int HoWo = p.Ho * p.Wo;
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
        const int c = tid + it * NT;
        const int m = m_base + c / CPR;
        a_ok[it] = (c < A_CH) && (m < p.M);
        const int mm = a_ok[it] ? m : 0;
        const int b = mm / HoWo, r = mm - b * HoWo;
        const int oh = r / p.Wo, ow = r - oh * p.Wo;
        a_base[it] = (unsigned)b * (unsigned)(p.H * p.W * p.Cin) * 2u;
        a_ih0[it] = oh * p.stride - p.pad;
        a_iw0[it] = ow * p.stride - p.pad;
    }
    bool b_ok[B_IT];
    unsigned b_base[B_IT];
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
        const int c = tid + it * NT;
        const int n = n_base + c / CPR;
        b_ok[it] = (c < B_CH) && (n < p.N);
        b_base[it] = (unsigned)(b_ok[it] ? n : 0) * (unsigned)p.K * 2u;
    }
    const int kc = (tid % CPR) * 8;          // same for every chunk of this thread: NT % CPR == 0
    const bool pointwise = (p.KH * p.KW == 1);

    auto load_tile = [&](int kt, uint4 (&ra)[A_IT], uint4 (&rb)[B_IT]) {
        const int k = kt * BK + kc;
        const bool k_ok = k < p.K;
        int kh = 0, kw = 0, ci = k;
        if (!pointwise) {
            const int tap = k / p.Cin;
            ci = k - tap * p.Cin;
            kh = tap / p.KW;
            kw = tap - kh * p.KW;
        }
#pragma unroll
        for (int it = 0; it < A_IT; ++it) {
            const int ih = a_ih0[it] + kh, iw = a_iw0[it] + kw;
            const bool ok = a_ok[it] && k_ok && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
            const unsigned off = ok ? a_base[it] + (unsigned)((ih * p.W + iw) * p.Cin + ci) * 2u : OOB;
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rx, off, 0, 0);
            ra[it] = make_uint4(v.x, v.y, v.z, v.w);
        }
#pragma unroll
        for (int it = 0; it < B_IT; ++it) {
            const unsigned off = (b_ok[it] && k_ok) ? b_base[it] + (unsigned)k * 2u : OOB;
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rw, off, 0, 0);
            rb[it] = make_uint4(v.x, v.y, v.z, v.w);
        }
    };
    auto store_tile = [&](int slot, const uint4 (&ra)[A_IT], const uint4 (&rb)[B_IT]) {
#pragma unroll
        for (int it = 0; it < A_IT; ++it) {
            const int c = tid + it * NT;
            if (c < A_CH) *reinterpret_cast<uint4 *>(&sA0[slot * BM * LDK + (c / CPR) * LDK + kc]) = ra[it];
        }
#pragma unroll
        for (int it = 0; it < B_IT; ++it) {
            const int c = tid + it * NT;
            if (c < B_CH) *reinterpret_cast<uint4 *>(&sB0[slot * BN * LDK + (c / CPR) * LDK + kc]) = rb[it];
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

    // RS register sets: set (t - kt_begin) % RS carries K step t, so RS steps of loads are in flight
    uint4 ra[RS][A_IT], rb[RS][B_IT];
#pragma unroll
    for (int r = 0; r < RS; ++r) load_tile(kt_begin + r < kt_end ? kt_begin + r : p.KT, ra[r], rb[r]);

    auto compute = [&](int slot) {
#pragma unroll
        for (int ks = 0; ks < BK / 32; ++ks) {
            uint4 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const uint4 *>(&sA0[slot * BM * LDK + (wm * (BM / WM) + i * 16 + frag_row) * LDK + ks * 32 + frag_k]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const uint4 *>(&sB0[slot * BN * LDK + (wn * (BN / WN) + j * 16 + frag_row) * LDK + ks * 32 + frag_k]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = Mma<T>::run(fb[j], fa[i], acc[i][j]);
        }
    };

    // LDS slot (t - kt_begin) % 2 is rewritten at step t only after every wavefront has passed the barrier
    // of step t-1, i.e. after all of them finished reading it at step t-2.  RS is even, so the slot of
    // register set r is r % 2.
    // The loop body is branch-free: steps at or beyond kt_end load zeros (k >= K in load_tile's terms is
    // forced by passing KT) and multiply them, which costs at most RS-1 idle steps at the end of a slice
    // and lets the compiler wait for exactly one step's loads at a time.
    if constexpr (!OVERLAP) {
        for (int kt = kt_begin; kt < kt_end; kt += RS) {
#pragma unroll
            for (int r = 0; r < RS; ++r) {
                store_tile(r & 1, ra[r], rb[r]);
                __syncthreads();
                const int nxt = kt + r + RS;
                load_tile(nxt < kt_end ? nxt : p.KT, ra[r], rb[r]);
                compute(r & 1);
            }
        }
    } else {
        // Large tiles (RS == 2): the LDS stores of step t+1 share a basic block with the MFMAs of step t, so
        // the scheduler can hide them behind the matrix pipe.  Safe with two slots: slot (t+1)%2 was last read
        // at step t-1, and every wavefront has passed the barrier that ended that step.
        static_assert(!OVERLAP || RS == 2, "the overlapped loop alternates two register sets");
        store_tile(0, ra[0], rb[0]);
        __syncthreads();
        for (int kt = kt_begin; kt < kt_end; kt += 2) {
            load_tile(kt + 2 < kt_end ? kt + 2 : p.KT, ra[0], rb[0]);
            compute(0);
            store_tile(1, ra[1], rb[1]);
            __syncthreads();
            load_tile(kt + 3 < kt_end ? kt + 3 : p.KT, ra[1], rb[1]);
            compute(1);
            store_tile(0, ra[0], rb[0]);
            __syncthreads();
        }
    }

    // lane owns output pixel m0 + (lane & 15) and channels n0 + 4*(lane >> 4) .. +3 of each 16x16 block
    const int m_l = m_base + wm * (BM / WM) + (lane & 15);
    const int n_l = n_base + wn * (BN / WN) + (lane >> 4) * 4;

    if (p.splits == 1) {
        static_for<TM>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            static_for<TN>([&](auto jc) {
                constexpr int j = decltype(jc)::value;
                epilogue_store<T>(p.bias, p.res, p.y, p.y32, p.M, p.N, p.act, m_l + i * 16, n_l + j * 16, acc[i][j]);
            });
        });
        return;
    }
    // split-K: this slice's partial sums go to ws[z][m][n]; a second kernel adds the slices.  (A single-kernel
    // form, in which the last slice to arrive at a per-tile counter does the sum, was measured and dropped:
    // across XCDs it needs either a device-scope fence, i.e. a write-back of the issuing XCD's whole L2 per
    // workgroup, or write-through stores and cache-bypassing loads for every partial sum; both cost several
    // times the second launch.)
    const bool vec = ((p.N & 3) == 0);
    static_for<TM>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        static_for<TN>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            const int m = m_l + i * 16, n = n_l + j * 16;
            if (m < p.M && n < p.N) {
                float *dst = p.ws + ((long)z * p.M + m) * p.N + n;
                if (vec) {
                    *reinterpret_cast<float4 *>(dst) = make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (n + r < p.N) dst[r] = acc[i][j][r];
                }
            }
        });
    });
}

// y = act(sum_z ws[z] + bias + res): one thread per 4 consecutive channels (one channel when N % 4 != 0).
// The slices are read eight at a time so that their loads overlap; the additions keep slice order.
template <typename T>
__global__ __launch_bounds__(64) void splitk_reduce_kernel(const float *ws, int splits, int M, int N, const uint16_t *bias,
                                                           const uint16_t *res, uint16_t *y, float *y32, int act)
{
    const bool vec = ((N & 3) == 0);
    const int per_row = vec ? N / 4 : N;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)M * per_row) return;
    const int m = (int)((unsigned)idx / (unsigned)per_row);
    const int n = (int)((unsigned)idx % (unsigned)per_row) * (vec ? 4 : 1);
    const long slice = (long)M * N;
    const float *src = ws + (long)m * N + n;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (vec) {
        for (int z0 = 0; z0 < splits; z0 += 8) {
            float4 q[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                q[u] = (z0 + u < splits) ? *reinterpret_cast<const float4 *>(src + (long)(z0 + u) * slice) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int u = 0; u < 8; ++u) { s[0] += q[u].x; s[1] += q[u].y; s[2] += q[u].z; s[3] += q[u].w; }
        }
    } else {
        for (int z = 0; z < splits; ++z) s[0] += src[z * slice];
    }
    epilogue_store<T>(bias, res, y, y32, M, N, act, m, n, s, vec ? 4 : 1);
}

struct Variant { int bm, bn, bk; };
constexpr Variant kVariants[4] = {{128, 128, 32}, {64, 64, 64}, {32, 64, 64}, {256, 256, 32}};

constexpr size_t lds_bytes(int bm, int bn, int bk) { return (size_t)2 * (bm + bn) * (bk + 8) * 2; }

template <typename T>
hipError_t launch_t(const GemmDev &d, const GemmPlan &pl, hipStream_t s)
{
    const dim3 grid((unsigned)pl.tiles, (unsigned)pl.splits);
    switch (pl.variant) {
    case 0: hipLaunchKernelGGL((conv_gemm_kernel<T, 128, 128, 32, 2, 2, 2>), grid, dim3(256), lds_bytes(128, 128, 32), s, d); break;
    case 1: hipLaunchKernelGGL((conv_gemm_kernel<T, 64, 64, 64, 2, 2, 4>), grid, dim3(256), lds_bytes(64, 64, 64), s, d); break;
    case 2: hipLaunchKernelGGL((conv_gemm_kernel<T, 32, 64, 64, 1, 4, 4>), grid, dim3(256), lds_bytes(32, 64, 64), s, d); break;
    default: hipLaunchKernelGGL((conv_gemm_kernel<T, 256, 256, 32, 2, 4, 2, true>), grid, dim3(512), lds_bytes(256, 256, 32), s, d); break;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.splits == 1) return e;
    const long threads = (long)d.M * ((d.N & 3) == 0 ? d.N / 4 : d.N);
    hipLaunchKernelGGL((splitk_reduce_kernel<T>), dim3((unsigned)((threads + 63) / 64)), dim3(64), 0, s, d.ws, pl.splits, d.M, d.N,
                       d.bias, d.res, d.y, d.y32, d.act);
    return hipGetLastError();
}

}  // namespace

hipError_t conv_gemm_init()
{
    hipError_t e = hipFuncSetAttribute((const void *)conv_gemm_kernel<bf16_t, 256, 256, 32, 2, 4, 2, true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds_bytes(256, 256, 32));
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute((const void *)conv_gemm_kernel<f16_t, 256, 256, 32, 2, 4, 2, true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)lds_bytes(256, 256, 32));
}

void conv_gemm_tile(int variant, int *bm, int *bn, int *bk)
{
    const int v = variant < 0 ? 0 : (variant > 3 ? 3 : variant);
    *bm = kVariants[v].bm;
    *bn = kVariants[v].bn;
    *bk = kVariants[v].bk;
}

static long cdiv(long a, long b) { return (a + b - 1) / b; }

// Large un-split problems are launched on the 8 x 4 block raster: the grid grows to whole blocks, 8 at a time.
static void set_raster(GemmPlan &pl, long M, long N)
{
    int bm, bn, bk;
    conv_gemm_tile(pl.variant, &bm, &bn, &bk);
    const long tm = cdiv(M, bm), tn = cdiv(N, bn);
    if (pl.kind != 0 || pl.splits != 1 || tm * tn < 256) return;
    const long blocks = cdiv(tm, 8) * cdiv(tn, 4);
    pl.raster = 1;
    pl.tiles = (int)(cdiv(blocks, 8) * 8 * 32);
}

GemmPlan conv_gemm_plan(long M, long N, long K, int n_cu, size_t ws_floats)
{
    auto tiles = [&](int v) { int bm, bn, bk; conv_gemm_tile(v, &bm, &bn, &bk); return cdiv(M, bm) * cdiv(N, bn); };
    auto wsk_tiles = [&](int v) { int bm, bn; conv_wsk_tile(v, &bm, &bn); return cdiv(M, bm) * cdiv(N, bn); };
    GemmPlan pl{0, 1, 1, 0, 4, 0};
    // tuning aid: ECLIP_GEMM_FORCE="kind,variant,n" overrides the heuristic; n = K splits (kind 0, clamped to the
    // workspace) or wavefronts per workgroup (kind 1: 4, 8 or 16)
    const char *force = getenv("ECLIP_GEMM_FORCE");
    int f_kind = -1, f_variant = -1, f_n = -1;
    if (force) sscanf(force, "%d,%d,%d", &f_kind, &f_variant, &f_n);
    if (f_kind == 1 && f_variant >= 0 && f_variant <= 2 && (f_n == 4 || f_n == 8 || f_n == 16) &&
        conv_wsk_lds_bytes(f_variant, f_n) <= 128 * 1024) {
        pl.kind = 1; pl.variant = f_variant; pl.nw = f_n; pl.tiles = (int)wsk_tiles(f_variant);
        return pl;
    }
    if (f_kind == 0 && f_variant >= 0 && f_variant <= 3) {
        pl.variant = f_variant;
        pl.tiles = (int)tiles(pl.variant);
        int bm, bn, bk;
        conv_gemm_tile(pl.variant, &bm, &bn, &bk);
        const long KT = cdiv(K, bk);
        long s = f_n < 1 ? 1 : f_n;
        if (s > KT) s = KT;
        while (s > 1 && (size_t)(s * M * N) > ws_floats) --s;
        const long kt_per = cdiv(KT, s);
        pl.splits = (int)cdiv(KT, kt_per);
        set_raster(pl, M, N);
        return pl;
    }
    // Few tiles (batch-1 convolutions, skinny linear layers).  Measured on MI355X: a kernel costs about
    // 4.5 us however little it does, and one CU sustains only about 30 GB/s of operand loads, so a layer is
    // priced as  launches * 4.5 us + (bytes the busiest CU has to pull) / 30 GB/s  for each candidate:
    //   wave-split-K on 16x64 or 32x64 tiles (one launch, a workgroup pulls its whole (bm+bn) x K panel);
    //   32x64 tiles cut along K over the grid (two launches, the panels are spread over every CU).
    if (wsk_tiles(1) <= 2L * n_cu) {
        const double us_per_launch = 4.5, bytes_per_us = 30e3;
        auto wsk_cost = [&](int v) {
            int bm, bn;
            conv_wsk_tile(v, &bm, &bn);
            const double rounds = (double)cdiv(wsk_tiles(v), n_cu);
            return us_per_launch + rounds * (double)(bm + bn) * (double)K * 2.0 / bytes_per_us;
        };
        const long t2 = tiles(2);
        const long KT = cdiv(K, 64);
        long s = 1;
        if (KT >= 8) {
            s = cdiv(2L * n_cu, t2);                   // about two workgroups per CU
            const long max_s = KT / 2;
            if (s > max_s) s = max_s;
            if (s > 32) s = 32;
            while (s > 1 && (size_t)(s * M * N) > ws_floats) --s;
        }
        const double split_cost = s > 1 ? 2.0 * us_per_launch + 0.5 +
                                              (double)cdiv(t2 * s, n_cu) * 96.0 * (double)cdiv(K, s) * 2.0 / bytes_per_us
                                        : 1e30;
        const int wv = (M <= 16 || wsk_cost(0) <= wsk_cost(1)) ? 0 : 1;
        if (split_cost < wsk_cost(wv)) {
            pl.kind = 0; pl.variant = 2; pl.tiles = (int)t2;
            const long kt_per = cdiv(KT, s);
            pl.splits = (int)cdiv(KT, kt_per);
            return pl;
        }
        pl.kind = 1;
        pl.variant = wv;
        pl.tiles = (int)wsk_tiles(wv);
        pl.nw = 4;
        return pl;
    }
    if (tiles(3) >= 2L * n_cu) pl.variant = 3;
    else if (tiles(0) >= 2L * n_cu) pl.variant = 0;
    else pl.variant = 1;
    pl.tiles = (int)tiles(pl.variant);
    set_raster(pl, M, N);
    return pl;
}

hipError_t launch_conv_gemm(const ConvGemmArgs &a, const GemmPlan &pl, hipStream_t s, uint32_t *n_launched)
{
    GemmDev d;
    d.x = (const uint16_t *)a.x; d.w = (const uint16_t *)a.w; d.bias = (const uint16_t *)a.bias;
    d.res = (const uint16_t *)a.res; d.y = (uint16_t *)a.y; d.y32 = a.y32; d.ws = a.ws;
    d.B = a.B; d.H = a.H; d.W = a.W; d.Cin = a.Cin; d.Ho = a.Ho; d.Wo = a.Wo; d.KH = a.KH; d.KW = a.KW;
    d.stride = a.stride; d.pad = a.pad; d.act = a.act;
    d.M = a.B * a.Ho * a.Wo; d.N = a.Cout; d.K = a.KH * a.KW * a.Cin;
    d.x_bytes = (unsigned)((size_t)a.B * a.H * a.W * a.Cin * 2);
    d.w_bytes = (unsigned)((size_t)d.N * d.K * 2);
    int bm, bn, bk;
    conv_gemm_tile(pl.variant, &bm, &bn, &bk);
    d.KT = (d.K + bk - 1) / bk;
    d.splits = pl.splits;
    d.kt_per = (d.KT + pl.splits - 1) / pl.splits;
    d.tiles_m = (d.M + bm - 1) / bm;
    d.tiles_n = (d.N + bn - 1) / bn;
    d.raster = pl.raster;
    if (n_launched) *n_launched += pl.splits > 1 ? 2 : 1;
    if (pl.kind == 1) {
        conv_wsk_tile(pl.variant, &bm, &bn);
        d.tiles_m = (d.M + bm - 1) / bm;
        return launch_conv_wsk(d, a.dtype, pl.variant, pl.nw, pl.tiles, s);
    }
    if (a.dtype == DT_BF16) return launch_t<bf16_t>(d, pl, s);
    return launch_t<f16_t>(d, pl, s);
}

}  // namespace eclip
