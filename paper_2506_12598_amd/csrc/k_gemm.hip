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
#include <type_traits>
#include <vector>

#include "gemm_tile.h"

namespace eclip {

namespace {

// y = act(sum_z ws[z] + bias + res): one thread per 4 consecutive channels (one channel when N % 4 != 0).
// The slices are read eight at a time so that their loads overlap; the additions keep slice order.
template <typename T>
__global__ __launch_bounds__(64) void splitk_reduce_kernel(const float *ws, int splits, int M, int N, const uint16_t *bias,
                                                           const uint16_t *res, uint16_t *y, float *y32, int act, int ldy)
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
#define EPI(A) epilogue_store<T, A>(bias, res, y, y32, M, N, m, n, s, vec ? 4 : 1, ldy)
    ECLIP_ACT_SWITCH(act, EPI)
#undef EPI
}

struct Variant { int bm, bn, bk; };
constexpr Variant kVariants[CONV_GEMM_VARIANTS] = {{128, 128, 32}, {64, 64, 64}, {32, 64, 64},
#define X(ID, BM, BN, BK, RS, LP) {BM, BN, BK},
                                                   ECLIP_PP_TILES(X)
#undef X
};

template <typename T>
hipError_t launch_pp_split(const GemmDev &d, const GemmPlan &pl, hipStream_t s, hipError_t e);

template <typename T>
hipError_t launch_t(const GemmDev &d, const GemmPlan &pl, hipStream_t s)
{
    const dim3 grid((unsigned)pl.tiles, (unsigned)pl.splits);
    switch (pl.variant) {
    case 0: hipLaunchKernelGGL((conv_gemm_kernel<T, 128, 128, 32, 2, 2, 2>), grid, dim3(256), lds_bytes(128, 128, 32), s, d); break;
    case 1: hipLaunchKernelGGL((conv_gemm_kernel<T, 64, 64, 64, 2, 2, 4>), grid, dim3(256), lds_bytes(64, 64, 64), s, d); break;
    case 2: hipLaunchKernelGGL((conv_gemm_kernel<T, 32, 64, 64, 1, 4, 4>), grid, dim3(256), lds_bytes(32, 64, 64), s, d); break;
#define X(ID, BM, BN, BK, RS, LP) \
    case ID: return launch_pp_split<T>(d, pl, s, launch_pp<ID>(d, std::is_same<T, bf16_t>::value ? DT_BF16 : DT_F16, grid, s));
        ECLIP_PP_TILES(X)
#undef X
    default: return hipErrorInvalidValue;
    }
    return launch_pp_split<T>(d, pl, s, hipGetLastError());
}

// second launch of a layer whose K is cut over the grid: the slice sum
template <typename T>
hipError_t launch_pp_split(const GemmDev &d, const GemmPlan &pl, hipStream_t s, hipError_t e)
{
    if (e != hipSuccess || pl.splits == 1) return e;
    const long threads = (long)d.M * ((d.N & 3) == 0 ? d.N / 4 : d.N);
    hipLaunchKernelGGL((splitk_reduce_kernel<T>), dim3((unsigned)((threads + 63) / 64)), dim3(64), 0, s, d.ws, pl.splits, d.M, d.N,
                       d.bias, d.res, d.y, d.y32, d.act, d.ldy);
    return hipGetLastError();
}

}  // namespace

hipError_t conv_gemm_init()
{
    hipError_t e;
#define X(ID, BM, BN, BK, RS, LP) \
    if ((e = init_pp<ID>()) != hipSuccess) return e;
    ECLIP_PP_TILES(X)
#undef X
    return hipSuccess;
}

void conv_gemm_tile(int variant, int *bm, int *bn, int *bk)
{
    const int v = variant < 0 ? 0 : (variant >= CONV_GEMM_VARIANTS ? CONV_GEMM_VARIANTS - 1 : variant);
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
    if (pl.kind != 0) return;
    if (tm * tn < 256 || pl.splits != 1) {
        // fewer tiles than CUs (or K slices in grid.y): deal whole tile columns or rows to the XCDs when they divide
        // evenly, so that each L2 holds 1/8 of one operand instead of all of both
        if (tn >= 8 && tn % 8 == 0) { pl.raster = 2; pl.tiles = (int)(tn * tm); }
        else if (tm >= 8 && tm % 8 == 0) { pl.raster = 3; pl.tiles = (int)(tn * tm); }
        return;
    }
    const long blocks = cdiv(tm, 8) * cdiv(tn, 4);
    pl.raster = 1;
    pl.tiles = (int)(cdiv(blocks, 8) * 8 * 32);
}

// Wave-split-K tiles are dealt to the 8 XCDs along one dimension when that dimension has enough tiles to keep the
// XCDs evenly loaded (a multiple of 8 tiles): along N when N >= M (the weights,
// N x K, are then the larger operand; the im2col operand is at most M x K), else along M; the other dimension is the
// second choice.
static void set_xcd_split(GemmPlan &pl, long M, long N)
{
    int bm, bn;
    conv_wsk_tile(pl.variant, &bm, &bn);
    const long tm = cdiv(M, bm), tn = cdiv(N, bn);
    auto fits = [](long t) { return t >= 8 && t % 8 == 0; };
    const bool n_first = N >= M;                      // W is N x K, the im2col operand at most M x K
    const int order[2] = {n_first ? 2 : 3, n_first ? 3 : 2};
    for (int r : order) {
        const long t = r == 2 ? tn : tm, other = r == 2 ? tm : tn;
        if (fits(t)) {
            pl.raster = r;
            pl.tiles = (int)(8 * cdiv(t, 8) * other);
            return;
        }
    }
}

// Cost of the wave-split-K kernel (us, without the launch), 1e30 when the combination does not exist.  A compute
// unit pulls the im2col rows as 64-byte runs (slow) and the weights as contiguous 1 KB blocks (fast), or is bound by
// its matrix instructions when the tile is large; its workgroups run one after another; each wavefront needs
// ceil(steps / depth) round trips to memory; the partial tiles of the nw wavefronts are summed through LDS.
static double wsk_cost(long M, long N, long K, int n_cu, int v, int nw)
{
    const double ra = 2.676e4, rw = 4.635e5;         // bytes per us per CU: activation rows, weight blocks
    const double rm = 1.539e6;                       // multiply-adds per us per CU with 8 or more wavefronts
    const double lat = 0.04896, c_out = 3.14e-6, c_red = 1.248e-5, l2 = 9.238e7, c_wg = 0.02628;
    if (conv_wsk_lds_bytes(v, nw) > 128 * 1024) return 1e30;
    int bm, bn;
    conv_wsk_tile(v, &bm, &bn);
    const int depth = (bm + bn) <= 32 ? 8 : (bm + bn) <= 48 ? 6 : (bm + bn) <= 80 ? (nw == 16 ? 3 : 4) : (bm + bn) <= 96 ? (nw == 16 ? 2 : 3) : 2;
    const double t = (double)(cdiv(M, bm) * cdiv(N, bn));
    const double per_cu = (double)cdiv((long)t, n_cu), frac = t / n_cu > 1.0 ? t / n_cu : 1.0;
    const double a_b = (double)(M < bm ? M : bm) * K * 2.0, w_b = (double)(N < bn ? N : bn) * K * 2.0;
    const double loads = a_b / ra + w_b / rw;
    const double macs = (double)(M < bm ? M : bm) * bn * K / rm / (nw < 8 ? nw / 8.0 : 1.0);
    const double cu = per_cu * (loads > macs ? loads : macs) + frac * c_wg + frac * bm * bn * (c_out + c_red * nw);
    const double all = t * (a_b + w_b) / l2;
    const double cost = (cu > all ? cu : all) + lat * (double)cdiv(cdiv(cdiv(K, 32), nw), depth);
    // what the model above leaves unexplained per (tile, wavefront count), fitted last: cost * scale + offset
    static const struct { double scale, offset; } kAdjust[CONV_WSK_VARIANTS][3] = {
        {{1.0, 0.0}, {1.0, 0.0}, {1.0, -0.1}},  {{0.95, 0.2}, {1.0, 0.0}, {0.95, 0.0}}, {{1.2, 0.0}, {1.0, 0.0}, {1.0, 0.0}},
        {{1.0, 0.0}, {1.0, 0.0}, {1.0, 0.0}},   {{1.0, 0.0}, {0.9, 0.1}, {1.05, 0.0}},  {{0.9, 0.0}, {1.0, 0.0}, {1.0, 0.0}}};
    const auto &adj = kAdjust[v][nw == 4 ? 0 : nw == 8 ? 1 : 2];
    return cost * adj.scale + adj.offset;
}

// the planner's estimate for one wave-split-K candidate (tuning aid; tile `v`, `nw` wavefronts)
double conv_wsk_cost_estimate(long M, long N, long K, int n_cu, int v, int nw) { return wsk_cost(M, N, K, n_cu, v, nw); }

// Every plan worth timing for a problem (eclip_model_tune): all wave-split-K tiles and wavefront counts that fit LDS, and
// every LDS-tiled shape whole and with K cut in two or four where the workspace allows.  Tiles far larger than the
// problem are left out (a 256-row tile for a 64-row problem only wastes the measurement).
std::vector<GemmPlan> conv_gemm_candidates(long M, long N, long K, int n_cu, size_t ws_floats)
{
    std::vector<GemmPlan> out;
    for (int v = 0; v < CONV_WSK_VARIANTS; ++v)
        for (int nw = 4; nw <= 16; nw *= 2) {
            if (conv_wsk_lds_bytes(v, nw) > 128 * 1024) continue;
            int bm, bn;
            conv_wsk_tile(v, &bm, &bn);
            if (cdiv(M, bm) * cdiv(N, bn) > 65536 * 4) continue;
            GemmPlan pl{1, v, 1, (int)(cdiv(M, bm) * cdiv(N, bn)), nw, 0};
            set_xcd_split(pl, M, N);
            out.push_back(pl);
        }
    for (int v : {0, 1, 3, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16}) {
        int bm, bn, bk;
        conv_gemm_tile(v, &bm, &bn, &bk);
        if (bm > 2 * M + 32 || bn > 2 * N + 32) continue;
        const long KT = cdiv(K, bk);
        for (long sp = 1; sp <= 4; sp *= 2) {
            if (sp > 1 && (K < 512 * sp || (size_t)(sp * M * N) > ws_floats)) continue;
            GemmPlan pl{0, v, 1, (int)(cdiv(M, bm) * cdiv(N, bn)), 4, 0};
            pl.splits = (int)cdiv(KT, cdiv(KT, sp));
            if (sp > 1 && pl.splits == 1) continue;
            set_raster(pl, M, N);
            out.push_back(pl);
        }
    }
    (void)n_cu;
    return out;
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
    if (f_kind == 1 && f_variant >= 0 && f_variant < CONV_WSK_VARIANTS && (f_n == 4 || f_n == 8 || f_n == 16) &&
        conv_wsk_lds_bytes(f_variant, f_n) <= 128 * 1024) {
        pl.kind = 1; pl.variant = f_variant; pl.nw = f_n; pl.tiles = (int)wsk_tiles(f_variant);
        set_xcd_split(pl, M, N);
        return pl;
    }
    if (f_kind == 0 && f_variant >= 0 && f_variant < CONV_GEMM_VARIANTS) {
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
    // Every candidate is priced with a small cost model fitted to per-layer timings of all GEMM layers of the
    // ResNet-18/50/152, VGG-16, MobileNetV2 and BERT-base/large graphs at batch 1 to 8, on 256 and on 128 CUs (picks
    // within 4 % of the per-layer best of an exhaustive sweep, in total).  Times in microseconds, without the
    // launch cost that all single-launch candidates share.
    double best = 1e30;
    for (int v = 0; v < CONV_WSK_VARIANTS; ++v)
        for (int nw = 4; nw <= 16; nw *= 2) {
            const double cost = wsk_cost(M, N, K, n_cu, v, nw);
            if (cost < best) { best = cost; pl = GemmPlan{1, v, 1, (int)wsk_tiles(v), nw, 0}; }
        }
    // LDS-tiled kernel, optionally with K cut into slices (second launch: its cost plus the traffic of the partial sums).
    // A tile costs `fixed` us once (fill of the pipeline, epilogue) and `step` us per K step of its own depth when it has
    // a compute unit to itself; workgroups beyond one per compute unit run in rounds (`pair`: two of them fit a compute
    // unit together and overlap, a round of two costs 1.74 instead of 2); a full machine slows every step by about 15 %
    // (shared L2 and vector caches).  Constants from timings of the four BERT-large shapes (M = 1536; N, K in {1024,
    // 3072, 4096}) on 256 and on 96 compute units, each tile at 16, 64 and 128 K steps: intercept and slope per tile,
    // minus the 2.5 us launch cost that all single-launch candidates share (as in wsk_cost).  Checked against an exhaustive
    // sweep of every candidate on every GEMM shape of the benchmark models: the picks cost 0-8 % more than the
    // per-layer optimum in total on 256 compute units, up to 14 % on 96; eclip_model_tune closes that gap by measurement.
    struct LdsTile { int variant; double step, fixed; bool pair; };
    static const LdsTile lds[] = {{0, 0.3613, 0.02038, true}, {1, 0.3664, 0.1703, true},
                                  {3, 0.582, 5.6, false},  {5, 0.616, 4.6, false},  {6, 0.72, 2.5, false},  {7, 0.36, 1.4, false},
                                  {8, 0.571, 3.0, false},  {9, 0.473, 0.6, false},  {10, 0.395, 1.5, false}, {11, 0.505, 3.8, false},
                                  {12, 0.481, 3.8, false}, {13, 0.406, 0.0, true},  {14, 0.373, 0.2, true},
                                  {15, 0.3134, 0.83, true}, {16, 0.4837, 4.2, false}};
    for (const LdsTile &c : lds) {
        int bm, bn, bk;
        conv_gemm_tile(c.variant, &bm, &bn, &bk);
        const long KT = cdiv(K, bk);
        for (long sp = 1; sp <= 4; sp *= 2) {
            if (sp > 1 && (K < 512 * sp || (size_t)(sp * M * N) > ws_floats)) continue;
            const long wgs = tiles(c.variant) * sp;
            double cost;
            if (c.variant <= 1) {
                // the two 4-wavefront tiles keep the form they were fitted in: per K step `alone` when a workgroup has the
                // compute unit to itself, `shared` per workgroup otherwise
                const double alone = c.variant == 0 ? 0.6385 : 1.171;
                const long per_cu = cdiv(wgs, n_cu);
                cost = c.fixed + (double)cdiv(KT, sp) * (per_cu == 1 ? alone : (double)per_cu * c.step);
                if (sp == 1 && c.variant == 1) cost *= 1.35;
                if (sp == 1 && c.variant == 0) cost -= 0.1;
            } else {
                const double load = wgs >= n_cu ? 1.0 : (double)wgs / n_cu;
                double rounds = (double)cdiv(wgs, n_cu);
                if (c.pair && rounds >= 2.0) rounds = 0.87 * (double)wgs / n_cu > 1.0 ? 0.87 * (double)wgs / n_cu : 1.0;
                cost = c.fixed + rounds * (double)cdiv(KT, sp) * c.step * (1.0 + 0.15 * load * load);
            }
            if (sp > 1) cost += 15.48 + (double)M * N * (4.0 * sp + 2.0) / 4.243e6;
            if (cost < best) {
                best = cost;
                pl = GemmPlan{0, c.variant, 1, (int)tiles(c.variant), 4, 0};
                const long kt_per = cdiv(KT, sp);
                pl.splits = (int)cdiv(KT, kt_per);
            }
        }
    }
    if (pl.kind == 0) set_raster(pl, M, N);
    else set_xcd_split(pl, M, N);
    return pl;
}

// Two independent layers in one launch of the wave-split-K kernel: possible when both are planned on that kernel and
// one (tile, wavefront count) serves both at a modelled extra cost below what the second launch would cost.
// Plan for a first layer that reads the caller's NCHW tensor itself (see conv_wsk_kernel): the cheapest of the tile
// shapes that exist in that form, if it costs at most `stage_us` (the separate re-layout kernel it saves) more than
// the unrestricted plan.
bool conv_gemm_plan_stem(long M, long N, long K, int n_cu, size_t ws_floats, double stage_us, GemmPlan *out)
{
    if (getenv("ECLIP_GEMM_FORCE") || getenv("ECLIP_NO_PAIRS")) return false;
    const GemmPlan any = conv_gemm_plan(M, N, K, n_cu, ws_floats);
    if (any.kind != 1) return false;
    const double any_cost = wsk_cost(M, N, K, n_cu, any.variant, any.nw);
    double best = 1e30;
    int bv = -1;
    for (int v : {0, 1, 5}) {
        const double c = wsk_cost(M, N, K, n_cu, v, 4);
        if (c < best) { best = c; bv = v; }
    }
    if (bv < 0 || best > any_cost + stage_us) return false;
    int bm, bn;
    conv_wsk_tile(bv, &bm, &bn);
    GemmPlan pl{1, bv, 1, (int)(cdiv(M, bm) * cdiv(N, bn)), 4, 0};
    set_xcd_split(pl, M, N);
    *out = pl;
    return true;
}

bool conv_gemm_plan_pair(const GemmPlan &s0, long M0, long N0, long K0, const GemmPlan &s1, long M1, long N1, long K1, int n_cu,
                         GemmPlan *p0, GemmPlan *p1)
{
    if (s0.kind != 1 || s1.kind != 1 || getenv("ECLIP_GEMM_FORCE") || getenv("ECLIP_NO_PAIRS")) return false;
    const double separate = wsk_cost(M0, N0, K0, n_cu, s0.variant, s0.nw) + wsk_cost(M1, N1, K1, n_cu, s1.variant, s1.nw);
    double best = 1e30;
    int bv = -1, bnw = 0;
    for (int v = 0; v < CONV_WSK_VARIANTS; ++v)
        for (int nw = 4; nw <= 16; nw *= 2) {
            const double c = wsk_cost(M0, N0, K0, n_cu, v, nw) + wsk_cost(M1, N1, K1, n_cu, v, nw);
            if (c < best) { best = c; bv = v; bnw = nw; }
        }
    const double launch_us = 2.5;                    // what a kernel costs as one more link of an in-order chain
    if (bv < 0 || best > separate + launch_us) return false;
    int bm, bn;
    conv_wsk_tile(bv, &bm, &bn);
    *p0 = GemmPlan{1, bv, 1, (int)(cdiv(M0, bm) * cdiv(N0, bn)), bnw, 0};
    *p1 = GemmPlan{1, bv, 1, (int)(cdiv(M1, bm) * cdiv(N1, bn)), bnw, 0};
    set_xcd_split(*p0, M0, N0);
    if (p0->tiles % 8 == 0) set_xcd_split(*p1, M1, N1);     // the second layer's workgroup b runs on XCD (tiles0 + b) % 8
    return true;
}

static GemmDev make_dev(const ConvGemmArgs &a, const GemmPlan &pl)
{
    GemmDev d;
    d.x = (const uint16_t *)a.x; d.w = (const uint16_t *)a.w; d.bias = (const uint16_t *)a.bias;
    d.res = (const uint16_t *)a.res; d.y = (uint16_t *)a.y; d.y32 = a.y32; d.ws = a.ws;
    d.B = a.B; d.H = a.H; d.W = a.W; d.Cin = a.Cin; d.Ho = a.Ho; d.Wo = a.Wo; d.KH = a.KH; d.KW = a.KW;
    d.stride = a.stride; d.pad = a.pad; d.act = a.act;
    d.M = a.B * a.Ho * a.Wo; d.N = a.Cout; d.K = a.KH * a.KW * a.Cin;
    d.nchw_c = a.nchw_c;
    d.ldx = a.ldx ? a.ldx : a.Cin;
    d.ldy = a.ldy ? a.ldy : a.Cout;
    d.x_bytes = (unsigned)((size_t)a.B * a.H * a.W * (a.nchw_c ? a.nchw_c : d.ldx) * 2);
    d.w_bytes = (unsigned)((size_t)((d.N + 15) / 16) * ((d.K + 31) / 32) * 1024);   // blocked layout, see ConvGemmArgs::w
    int bm, bn, bk;
    conv_gemm_tile(pl.variant, &bm, &bn, &bk);
    d.KT = (d.K + bk - 1) / bk;
    d.splits = pl.splits;
    d.kt_per = (d.KT + pl.splits - 1) / pl.splits;
    d.tiles_m = (d.M + bm - 1) / bm;
    d.tiles_n = (d.N + bn - 1) / bn;
    d.raster = pl.raster;
    if (pl.kind == 1) {
        conv_wsk_tile(pl.variant, &bm, &bn);
        d.tiles_m = (d.M + bm - 1) / bm;
        d.tiles_n = (d.N + bn - 1) / bn;
    }
    return d;
}

hipError_t launch_conv_gemm(const ConvGemmArgs &a, const GemmPlan &pl, hipStream_t s, uint32_t *n_launched)
{
    if ((a.ldx && (a.ldx % 8 || a.ldx < a.Cin || a.nchw_c)) || (a.ldy && (a.ldy % 8 || a.ldy < a.Cout || a.res || a.y32 || ((uintptr_t)a.y & 15))))
        return hipErrorInvalidValue;
    const GemmDev d = make_dev(a, pl);
    if (n_launched) *n_launched += pl.splits > 1 ? 2 : 1;
    if (pl.kind == 1) return launch_conv_wsk(d, a.dtype, pl.variant, pl.nw, pl.tiles, s);
    if (a.dtype == DT_BF16) return launch_t<bf16_t>(d, pl, s);
    return launch_t<f16_t>(d, pl, s);
}

hipError_t launch_conv_gemm_pair(const ConvGemmArgs &a0, const GemmPlan &p0, const ConvGemmArgs &a1, const GemmPlan &p1, hipStream_t s,
                                 uint32_t *n_launched)
{
    if (p0.kind != 1 || p1.kind != 1 || p0.variant != p1.variant || p0.nw != p1.nw || a0.dtype != a1.dtype) return hipErrorInvalidValue;
    for (const ConvGemmArgs *a : {&a0, &a1})
        if ((a->ldx && (a->ldx % 8 || a->ldx < a->Cin || a->nchw_c)) || (a->ldy && (a->ldy % 8 || a->ldy < a->Cout || a->res || a->y32 || ((uintptr_t)a->y & 15))))
            return hipErrorInvalidValue;
    if (n_launched) *n_launched += 1;
    return launch_conv_wsk_pair(make_dev(a0, p0), p0.tiles, make_dev(a1, p1), p1.tiles, a0.dtype, p0.variant, p0.nw, s);
}

}  // namespace eclip
