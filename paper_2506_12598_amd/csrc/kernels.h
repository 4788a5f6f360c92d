// Host-callable launchers of the gfx950 kernels.  Every launcher validates nothing: the caller
// (the model loader) has already checked shapes, alignment and capacity.  Internal layout of all
// activations is channels-last: [B][H][W][C] for images, [B][S][Hd] for sequences, [B][n] for vectors.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

namespace eclip {

enum { DT_F32 = 0, DT_BF16 = 1, DT_F16 = 2 };

// ---- implicit-GEMM convolution / linear on the matrix cores (16-bit types) -------------------
// y[m][n] = act(sum_k A[m][k] * w[n][k] + bias[n] + res[m][n]),  m = (b,oh,ow), k = (kh,kw,ci).
struct ConvGemmArgs {
    const void *x;       // [B][H][W][Cin]           Cin % 8 == 0
    const void *w;       // W[n][k], n = cout, k = (kh, kw, ci), in 1 KB blocks of 16 n x 32 k: block (nb, kb) at
                         // (nb * ceil(K/32) + kb) * 1 KB, lane l of a block = W[16 nb + (l & 15)][32 kb + 8 (l >> 4) .. +7];
                         // rows beyond Cout and k beyond K are zero
    const void *bias;    // [Cout] or null
    const void *res;     // [M][Cout] or null
    void *y;             // [M][Cout] in the model dtype, or null when y32 is used
    float *y32;          // [M][Cout] float output, or null
    float *ws;           // split-K partial sums, >= splits*M*Cout floats when splits > 1
    int B, H, W, Cin, Ho, Wo, Cout, KH, KW, stride, pad, act, dtype;
    int nchw_c = 0;      // > 0: x is [B][nchw_c][H][W] with nchw_c <= 4 real channels, Cin == 8 (wave-split-K plans of conv_gemm_plan_stem only)
    int ldx = 0;         // > 0: elements between consecutive pixels of x (x is the first Cin channels of a wider tensor); a multiple of 8
    int ldy = 0;         // > 0: elements between consecutive rows of y (y points at a channel range of a wider tensor); a multiple of 8,
                         // y 16-byte aligned, res and y32 null
};
struct GemmPlan {
    int kind;      // 0 = LDS-tiled kernel (large problems), 1 = wave-split-K kernel (few tiles, long K)
    int variant;   // tile shape, see conv_gemm_tile() / conv_wsk_tile()
    int splits;    // kind 0: K is cut into this many slices, summed by a second kernel
    int tiles;     // output tiles = workgroups (per slice)
    int nw;        // kind 1: wavefronts per workgroup, each taking 1/nw of K
    int raster;    // kind 0: workgroups walk the tiles in 8 x 4 blocks per XCD (tiles then counts whole blocks)
};
bool conv_gemm_plan_stem(long M, long N, long K, int n_cu, size_t ws_floats, double stage_us, GemmPlan *out);   // ConvGemmArgs::nchw_c
enum { CONV_GEMM_VARIANTS = 17 };        // 0..2: 128x128x32, 64x64x64, 32x64x64 (4 wavefronts); 3, 4: 256x256x32, 128x256x64 (8 wavefronts on the
                                         // ping-pong schedule, both operands in LDS); 5..14: ping-pong with the weights straight from memory:
                                         // 256x256x32, 128x256x64, 192x128x32, 192x128x64, 128x128x64, 256x128x32, 192x256x32, 256x192x32,
                                         // 64x128x64, 128x64x64, 96x64x64, 96x192x64
void conv_gemm_tile(int variant, int *bm, int *bn, int *bk);
enum { CONV_WSK_VARIANTS = 6 };          // 16x64, 32x64, 64x64, 16x16, 16x32, 32x32
void conv_wsk_tile(int variant, int *bm, int *bn);
size_t conv_wsk_lds_bytes(int variant, int nw);
hipError_t conv_gemm_init();   // raises the dynamic LDS limit of the 256x256 tile once per process
hipError_t conv_wsk_init();    // raises the dynamic LDS limit of the wave-split-K kernels once per process
// Chooses tile shape and K split for a stream restricted to n_cu compute units.
GemmPlan conv_gemm_plan(long M, long N, long K, int n_cu, size_t ws_floats);
// every plan worth timing for a problem (measured plan selection)
std::vector<GemmPlan> conv_gemm_candidates(long M, long N, long K, int n_cu, size_t ws_floats);
double conv_wsk_cost_estimate(long M, long N, long K, int n_cu, int variant, int nw);   // the planner's estimate, us without the launch
// *n_launched (optional) is increased by the number of kernels launched (2 when K is split).
hipError_t launch_conv_gemm(const ConvGemmArgs &a, const GemmPlan &p, hipStream_t s, uint32_t *n_launched);
// Two layers that do not depend on each other in one launch (wave-split-K kernel only).  conv_gemm_plan_pair takes
// the layers' own plans and returns true, with a common plan for each, when sharing a launch is modelled to pay.
bool conv_gemm_plan_pair(const GemmPlan &s0, long M0, long N0, long K0, const GemmPlan &s1, long M1, long N1, long K1, int n_cu,
                         GemmPlan *p0, GemmPlan *p1);
hipError_t launch_conv_gemm_pair(const ConvGemmArgs &a0, const GemmPlan &p0, const ConvGemmArgs &a1, const GemmPlan &p1, hipStream_t s,
                                 uint32_t *n_launched);

// ---- float32 direct convolution / linear (plain FMA) -------------------------------------------
struct ConvF32Args {
    const float *x;      // [B][H][W][Cin]
    const float *w;      // [KH][KW][Cin][Cout]
    const float *bias, *res;
    float *y;            // [M][Cout]
    int B, H, W, Cin, Ho, Wo, Cout, KH, KW, stride, pad, act;
};
hipError_t launch_conv_f32(const ConvF32Args &a, hipStream_t s);

// ---- memory-bound kernels ---------------------------------------------------------------------
struct DwConvArgs {
    const void *x, *w, *bias, *res;   // x [B][H][W][C]; w [KH][KW][C]
    void *y;
    int B, H, W, C, Ho, Wo, KH, KW, stride, pad, act, dtype;
};
int dwconv_pixels_per_thread(const DwConvArgs &a, int n_cu);   // 4 (large 3x3 layers, 16-bit types) or 1
int dwconv_strip_rows(const DwConvArgs &a, int n_cu);          // rows per thread of the strip kernel, or 0
hipError_t launch_dwconv(const DwConvArgs &a, int n_cu, hipStream_t s);

// grouped convolution, 1 < groups < C: one thread per output element, weights [Cout][KH][KW][Cin/groups]
struct GConvArgs {
    const void *x, *w, *bias, *res;
    void *y;
    int B, H, W, Cin, Ho, Wo, Cout, KH, KW, stride, pad, groups, act, dtype;
};
hipError_t launch_gconv(const GConvArgs &a, int n_cu, hipStream_t s);
// The same on the matrix cores (k_gconv.hip): S neighbouring groups form a dense block-diagonal problem.  gconv_mfma_pick
// returns false when no S <= 16 dividing `groups` makes S*cig a multiple of 32 and S*cog a multiple of 16; the weights
// must then be in the direct kernel's layout, otherwise in the super-group blocks described in k_gconv.hip.
bool gconv_mfma_pick(int groups, int cig, int cog, int *S_out);
hipError_t launch_gconv_mfma(const GConvArgs &a, int S, int n_cu, hipStream_t s);
long gconv_mfma_workgroups(long M, int groups, int cog, int S, int n_cu);   // the grid launch_gconv_mfma uses (M = B*Ho*Wo)
// y[m][0 .. c0) = a[m][:], y[m][c0 .. c0 + c1) = b[m][:]
hipError_t launch_concat(const void *a, const void *b, void *y, long rows, int c0, int c1, int dtype, hipStream_t s);
// y[m][0 .. c) = x[m][:], rows of y ld channels apart (16-bit types, c and ld multiples of 8)
hipError_t launch_chancopy(const void *x, void *y, long rows, int c, int ld, int dtype, hipStream_t s);
// y[m][j] = x[m][(j % groups) * (c / groups) + j / groups]
hipError_t launch_shuffle(const void *x, void *y, long rows, int c, int groups, int dtype, hipStream_t s);

struct PoolArgs {
    const void *x; void *y;
    int B, H, W, C, Ho, Wo, KH, KW, stride, pad, dtype;
};
hipError_t launch_maxpool(const PoolArgs &a, int n_cu, hipStream_t s);
// mean over HW: x [B][HW][C] -> y [B][C] (model dtype) or y32 (float).  Large HW is cut into parts whose float sums
// go through ws (>= B*parts*C floats) and a second kernel; *n_launched grows by the kernels launched.
int gap_parts(int B, int HW, int C, int n_cu);
hipError_t launch_gap(const void *x, void *y, float *y32, float *ws, size_t ws_floats, int B, int HW, int C, int dtype, int n_cu,
                      hipStream_t s, uint32_t *n_launched);

// global average pool and the linear layer that follows it in one launch (small batch, moderate C x HW):
// x [B][HW][C], w in the blocked GEMM layout of an N x C matrix, y [B][N] (model dtype) or y32 (float)
bool gapfc_supported(int B, int HW, int C, int dtype);
hipError_t launch_gapfc(const void *x, const void *w_blocked, const void *bias, void *y, float *y32, int B, int HW, int C, int N, int act,
                        int dtype, hipStream_t s);

struct RowArgs {
    const void *x, *res, *gamma, *beta;
    void *y; float *y32;
    long rows; int width; float eps; int dtype;
};
hipError_t launch_layernorm(const RowArgs &a, int n_cu, hipStream_t s);
hipError_t launch_softmax(const RowArgs &a, int n_cu, hipStream_t s);

struct EltArgs {
    const void *x, *bias, *res; void *y; float *y32;
    long rows; int width; int act; int dtype;
};
hipError_t launch_eltwise(const EltArgs &a, int n_cu, hipStream_t s);

struct EmbedArgs {
    const int32_t *ids; const void *tok, *pos, *typ; void *y;
    int B, S, Hd, vocab, dtype;
};
hipError_t launch_embed(const EmbedArgs &a, int n_cu, hipStream_t s);

// ---- fused attention ---------------------------------------------------------------------------
struct AttnArgs {
    const void *qkv;     // [B][S][3*Hd]
    void *y; float *y32; // [B][S][Hd]
    int B, S, Hd, heads, dtype;
};
size_t attention_lds_bytes(int S, int d);
hipError_t launch_attention(const AttnArgs &a, int n_cu, hipStream_t s);
hipError_t attention_init();   // raises the dynamic LDS limit once per process

// ---- layout conversion at the model boundary ------------------------------------------------------
// [B][C][H][W] (model dtype) -> [B][H][W][Cp], channels C..Cp-1 zero
hipError_t launch_nchw_to_nhwc(const void *x, void *y, int B, int C, int H, int W, int Cp, int dtype, hipStream_t s);
// internal [B][H][W][C] -> float32 [B][C][H][W]
hipError_t launch_nhwc_to_nchw_f32(const void *x, float *y, int B, int C, int H, int W, int dtype, hipStream_t s);
// n elements of the model dtype -> float32
hipError_t launch_to_f32(const void *x, float *y, long n, int dtype, hipStream_t s);

// ---- diagnostics -------------------------------------------------------------------------------
hipError_t launch_probe(uint32_t *out, int n_blocks, hipStream_t s);
hipError_t launch_tick(uint32_t *p, hipStream_t s);
hipError_t launch_fill_u32(uint32_t *p, uint32_t v, long n, hipStream_t s);

}  // namespace eclip
