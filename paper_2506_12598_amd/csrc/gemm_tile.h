// The LDS-tiled matrix-core kernel (implicit-GEMM convolution / linear layer) and its epilogue, shared by the
// translation units that instantiate its tile shapes.  See k_gemm.hip for the description of the tiling.
#pragma once
#include "gemm_common.h"
#include "kernels.h"

namespace eclip {

// Epilogue of one workgroup tile: acc[i][j] is the 16x16 block (i, j) of the wavefront's sub-tile, lane l holding
// output pixel (l & 15) and channels 4 (l >> 4) .. +3 of the block.  `smem` is the workgroup's LDS (the K loop is
// done with it); z is the K slice.
template <typename T, int BM, int BN, int WM, int WN, int TM, int TN, int ACT, bool N8>
__device__ __forceinline__ void tile_epilogue_impl(const GemmDev &p, f32x4 (&acc)[TM][TN], uint16_t *smem, int m_base, int n_base, int z)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    if (p.splits == 1) {
        // Row-contiguous stores.  Straight out of the accumulators a store instruction would write 8 bytes to each
        // of 64 different rows (measured: 6.4 us for the 12.6 MB output of a 1536 x 4096 layer, 2 TB/s).  Instead
        // each wavefront passes its sub-tile through a private LDS buffer, 32 rows at a time, and writes 16 bytes
        // (8 channels) per lane along the rows: whole 128-byte lines, and the bias and residual reads get the same
        // shape.  The buffer is private to the wavefront, so after the one barrier that ends the K loop's use of
        // LDS only the wavefront's own LDS counter is waited on.  N8: N is a multiple of 8, so a lane's 8 channels
        // are all inside the row and aligned; otherwise the (rare) ragged form stores them one by one from a loop
        // that is not unrolled, to keep it out of the way.
        // 32 rows (two 16-row blocks) per round; an odd TM ends with a round of 16
        if constexpr (N8 && TN % 2 == 0) {
            // Even TN: no LDS at all.  The four lanes that hold a pixel's channels of two neighbouring blocks (quads
            // q = lane >> 4 of blocks j and j + 1) trade registers so that each ends up with 8 consecutive channels:
            // v_permlane16_swap exchanges the odd 16-lane rows of one register with the even rows of another, which
            // leaves lane row q with channels 16 (q & 1) + 8 (q >> 1) .. +7 of the 32-channel pair.  A store
            // instruction then writes 16 bytes per lane, 64 contiguous bytes per pixel.  Bias and residual are fetched
            // before the first store, as below.
            const int q = lane >> 4;
            const int m0 = m_base + wm * (BM / WM) + (lane & 15);
            const int n0 = n_base + wn * (BN / WN) + 16 * (q & 1) + 8 * (q >> 1);
            float bv[TN / 2][8];
            uint4 rq[TM][TN / 2];
            static_for<TN / 2>([&](auto jc) {
                constexpr int jp = decltype(jc)::value;
#pragma unroll
                for (int e = 0; e < 8; ++e) bv[jp][e] = 0.f;
                if (p.bias && n0 + 32 * jp < p.N) Pack<T, 8>::load(reinterpret_cast<const T *>(p.bias) + n0 + 32 * jp, bv[jp]);
            });
            if (p.res) {
                static_for<TM>([&](auto ic) {
                    constexpr int i = decltype(ic)::value;
                    static_for<TN / 2>([&](auto jc) {
                        constexpr int jp = decltype(jc)::value;
                        const int m = m0 + 16 * i, n = n0 + 32 * jp;
                        rq[i][jp] = (m < p.M && n < p.N) ? *reinterpret_cast<const uint4 *>(p.res + (long)m * p.ldy + n) : make_uint4(0u, 0u, 0u, 0u);
                    });
                });
            }
            static_for<TM>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                static_for<TN / 2>([&](auto jc) {
                    constexpr int jp = decltype(jc)::value;
                    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
                    float o[8];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const u32x2 sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(acc[i][2 * jp][c]), __float_as_uint(acc[i][2 * jp + 1][c]), false, false);
                        o[c] = __uint_as_float(sw[0]);
                        o[4 + c] = __uint_as_float(sw[1]);
                    }
                    const int m = m0 + 16 * i, n = n0 + 32 * jp;
                    if (m < p.M && n < p.N) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) o[e] += bv[jp][e];
                        if (p.res) {
                            const uint32_t w[4] = {rq[i][jp].x, rq[i][jp].y, rq[i][jp].z, rq[i][jp].w};
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                o[2 * e] += Cvt<T>::from_bits(w[e] & 0xffffu);
                                o[2 * e + 1] += Cvt<T>::from_bits(w[e] >> 16);
                            }
                        }
                        epilogue_store8<T, ACT>(nullptr, nullptr, p.y, p.y32, p.ldy, m, n, o);
                    }
                });
            });
            return;
        }
        constexpr int COLS = TN * 16, SP = COLS + 4;          // row pitch in floats: the 4-float pad spreads the banks
        constexpr int LPR = COLS / 8, RPP = 64 / LPR;          // lanes per row, rows per pass (lanes beyond RPP * LPR idle)
        constexpr int PASSES = (32 + RPP - 1) / RPP;
        __syncthreads();
        float *stage = reinterpret_cast<float *>(smem) + wave * (32 * SP);
        const int rr0 = lane / LPR, col8 = (lane % LPR) * 8;
        const int n = n_base + wn * (BN / WN) + col8;
        constexpr int ROUNDS = (TM + 1) / 2;
        const int m0 = m_base + wm * (BM / WM) + rr0;
        // Everything the rounds read from global memory is fetched here, before their first store: a lane's 8 channels
        // are the same in every pass, so the bias is read once, and the residual chunks of all passes are in flight
        // together.  Loaded inside the passes, each read would queue behind the previous pass's store (loads and stores
        // retire in issue order, and the compiler cannot move a load across a store that may alias it): sixteen
        // dependent round trips on a 256 x 256 tile, about 10 us against 2 for the stores themselves.
        float bv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        uint4 rq[ROUNDS][PASSES];
        if constexpr (N8) {
            if (p.bias && n < p.N) Pack<T, 8>::load(reinterpret_cast<const T *>(p.bias) + n, bv);
            if (p.res) {
                static_for<ROUNDS>([&](auto hc) {
                    constexpr int h = decltype(hc)::value;
                    constexpr int NBLK = (2 * h + 1 < TM) ? 2 : 1;
                    static_for<PASSES>([&](auto pc) {
                        constexpr int ps = decltype(pc)::value;
                        const int rr = ps * RPP + rr0, m = m0 + h * 32 + ps * RPP;
                        const bool ok = lane < RPP * LPR && rr < NBLK * 16 && m < p.M && n < p.N;
                        rq[h][ps] = ok ? *reinterpret_cast<const uint4 *>(p.res + (long)m * p.ldy + n) : make_uint4(0u, 0u, 0u, 0u);
                    });
                });
            }
        }
        static_for<ROUNDS>([&](auto hc) {
            constexpr int h = decltype(hc)::value;
            constexpr int NBLK = (2 * h + 1 < TM) ? 2 : 1;       // 16-row blocks in this round
            static_for<NBLK>([&](auto ic) {
                constexpr int i2 = decltype(ic)::value;
                static_for<TN>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
                    const f32x4 a4 = acc[2 * h + i2][j];
                    *reinterpret_cast<float4 *>(&stage[(i2 * 16 + (lane & 15)) * SP + j * 16 + (lane >> 4) * 4]) = make_float4(a4[0], a4[1], a4[2], a4[3]);
                });
            });
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_s_waitcnt(0xc07f);              // lgkmcnt(0): this wavefront's LDS writes have landed
            if constexpr (N8) {
                static_for<PASSES>([&](auto pc) {
                    constexpr int ps = decltype(pc)::value;
                    const int rr = ps * RPP + rr0, m = m0 + h * 32 + ps * RPP;
                    if (lane < RPP * LPR && rr < NBLK * 16 && m < p.M && n < p.N) {
                        const float4 q0 = *reinterpret_cast<const float4 *>(&stage[rr * SP + col8]);
                        const float4 q1 = *reinterpret_cast<const float4 *>(&stage[rr * SP + col8 + 4]);
                        float o[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
#pragma unroll
                        for (int e = 0; e < 8; ++e) o[e] += bv[e];
                        if (p.res) {
                            const uint32_t w[4] = {rq[h][ps].x, rq[h][ps].y, rq[h][ps].z, rq[h][ps].w};
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                o[2 * e] += Cvt<T>::from_bits(w[e] & 0xffffu);
                                o[2 * e + 1] += Cvt<T>::from_bits(w[e] >> 16);
                            }
                        }
                        epilogue_store8<T, ACT>(nullptr, nullptr, p.y, p.y32, p.ldy, m, n, o);
                    }
                });
            } else {
#pragma unroll 1
                for (int ps = 0; ps < PASSES; ++ps) {
                    const int rr = ps * RPP + rr0, m = m0 + h * 32 + ps * RPP;
                    if (lane < RPP * LPR && rr < NBLK * 16 && m < p.M && n < p.N) {
                        const float4 q0 = *reinterpret_cast<const float4 *>(&stage[rr * SP + col8]);
                        const float4 q1 = *reinterpret_cast<const float4 *>(&stage[rr * SP + col8 + 4]);
                        const float o[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
                        epilogue_store8_ragged<T, ACT>(p.bias, p.res, p.y, p.y32, p.N, p.ldy, m, n, o);
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_s_waitcnt(0xc07f);              // reads done before the next 32 rows overwrite the buffer
        });
        return;
    }
    // lane owns output pixel m0 + (lane & 15) and channels n0 + 4*(lane >> 4) .. +3 of each 16x16 block
    const int m_l = m_base + wm * (BM / WM) + (lane & 15);
    const int n_l = n_base + wn * (BN / WN) + (lane >> 4) * 4;
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
template <typename T, int BM, int BN, int WM, int WN, int TM, int TN>
__device__ __forceinline__ void tile_epilogue(const GemmDev &p, f32x4 (&acc)[TM][TN], uint16_t *smem, int m_base, int n_base, int z)
{
    // the partial sums of a K slice take no activation
    if (p.splits != 1) { tile_epilogue_impl<T, BM, BN, WM, WN, TM, TN, ACT_NONE, true>(p, acc, smem, m_base, n_base, z); return; }
    if ((p.N & 7) == 0) {
#define EPI(A) tile_epilogue_impl<T, BM, BN, WM, WN, TM, TN, A, true>(p, acc, smem, m_base, n_base, z)
        ECLIP_ACT_SWITCH(p.act, EPI)
#undef EPI
    } else {
#define EPI(A) tile_epilogue_impl<T, BM, BN, WM, WN, TM, TN, A, false>(p, acc, smem, m_base, n_base, z)
        ECLIP_ACT_SWITCH(p.act, EPI)
#undef EPI
    }
}

// K-loop schedules
enum { LOOP_PLAIN = 0, LOOP_PINGPONG = 2, LOOP_PP_BDIRECT = 3 };

// How the im2col operand is addressed along K (chosen per launch from the layer's shape):
//   A_GENERAL  any window, any channel count: every thread tracks the (kh, kw, ci) position of its own chunk
//   A_UNIFORM  Cin is a multiple of BK: a K step never straddles two window taps, so the tap and the channel
//              base are the same for the whole workgroup and live in scalar registers; a thread adds its constant
//              offset and checks the image borders
//   A_MATRIX   1x1 window and K a multiple of BK (linear layers, pointwise convolutions): the operand is a matrix
//              with contiguous rows; every thread's offsets are constants and the position along K is one scalar
//              handed to the load instruction as its scalar offset -- no vector arithmetic in the K loop at all
// Counters on the general form showed 135 vector instructions per K step and wavefront next to 24 matrix
// instructions (the vector pipe busier than the matrix pipe); the specialised forms are what the large layers run.
enum { A_GENERAL = 0, A_UNIFORM = 1, A_MATRIX = 2 };

template <typename T, int BM, int BN, int BK, int WM, int WN, int RS, int LOOP = LOOP_PLAIN, int AMODE = A_GENERAL>
__global__ __launch_bounds__(WM * WN * 64) void conv_gemm_kernel(GemmDev p)
{
    constexpr int NT = WM * WN * 64;         // threads per workgroup: 4 wavefronts, 8 for the 256x256 tile
    static_assert(RS % 2 == 0, "register stages alternate between the two LDS slots");
    // row pitch in elements.  Measured with a ds_read_b128 / ds_write_b128 micro-benchmark: with 64-byte rows a
    // pitch of 96 bytes makes the fragment reads (16 rows x 4 chunks per instruction) conflict-free, 80 bytes
    // costs them about 20 %.
    constexpr bool BDIR = LOOP == LOOP_PP_BDIRECT;      // the weights bypass LDS (see the K loop below)
    constexpr int LDK = (LOOP == LOOP_PINGPONG || BDIR) ? BK + 16 : BK + 8;
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
    if (p.raster == 2) {                      // an XCD owns a contiguous range of tile columns (mid-size problems)
        const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3, per = (p.tiles_n + 7) >> 3, r = q / p.tiles_m;
        tile_m = q - r * p.tiles_m;
        tile_n = xcd * per + r;
        if (r >= per || tile_n >= p.tiles_n) return;
    } else if (p.raster == 3) {               // ... or of tile rows
        const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3, per = (p.tiles_m + 7) >> 3, r = q / p.tiles_n;
        tile_n = q - r * p.tiles_n;
        tile_m = xcd * per + r;
        if (r >= per || tile_m >= p.tiles_m) return;
    } else if (p.raster) {
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
    const int m_base = tile_m * BM, n_base = tile_n * BN;

    // ---- per-thread, per-chunk addressing that does not change along K
    // Operands are read through buffer descriptors: a lane whose chunk is padding, beyond M / N or beyond K
    // is given an offset past the end of the buffer, for which the hardware returns zeros.  This keeps the
    // loads free of branches, so the loads of different K steps are counted apart by the hardware.
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, (int)p.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void *)p.w, 0, (int)p.w_bytes, 0x00020000);
    constexpr unsigned OOB = 0xffffffffu;
    bool a_ok[A_IT];
    unsigned a_off0[A_IT];                   // byte offset of pixel (ih0, iw0) of the row's image (modulo 2^32 when padded)
    int a_ih0[A_IT], a_iw0[A_IT];
    const int HoWo = p.Ho * p.Wo;
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
        const int c = tid + it * NT;
        const int m = m_base + c / CPR;
        a_ok[it] = (A_CH % NT == 0 || c < A_CH) && (m < p.M);
        const int mm = a_ok[it] ? m : 0;
        const int b = mm / HoWo, r = mm - b * HoWo;
        const int oh = r / p.Wo, ow = r - oh * p.Wo;
        a_ih0[it] = oh * p.stride - p.pad;
        a_iw0[it] = ow * p.stride - p.pad;
        a_off0[it] = ((unsigned)b * (unsigned)(p.H * p.W) + (unsigned)(a_ih0[it] * p.W + a_iw0[it])) * (unsigned)p.ldx * 2u;
    }
    // The weights are stored in blocks of 16 rows x 32 k, 1 KB each, lane-ordered for the matrix instruction.  A
    // wavefront copies whole blocks: chunk c of the tile is lane c % 64 of block c / 64, and block b of the tile is
    // (row block b / (BK/32), k block b % (BK/32)).  Padding rows and k are zeros in memory, so the only checks are
    // the end of the matrix and the end of this workgroup's K slice.
    static_assert(NT % 64 == 0 && BK % 32 == 0 && BN % 16 == 0, "whole weight blocks per wavefront");
    constexpr int KBT = BK / 32;             // k blocks per tile
    const int KB = (p.K + 31) >> 5, NB = (p.N + 15) >> 4;
    bool b_ok[B_IT];
    unsigned b_base[B_IT];                   // byte offset of this lane's 16 bytes in k block 0 of its row block
    int b_kb[B_IT];                          // k block within the tile
    int b_lds[B_IT];                         // element offset in the LDS tile
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
        const int c = tid + it * NT;
        const int blk = c >> 6, nbl = blk / KBT;
        b_kb[it] = blk - nbl * KBT;
        const int nb = (n_base >> 4) + nbl;
        b_ok[it] = (B_CH % NT == 0 || c < B_CH) && (nb < NB);
        b_base[it] = ((unsigned)(b_ok[it] ? nb : 0) * (unsigned)KB * 64u + (unsigned)lane) * 16u;
        b_lds[it] = (nbl * 16 + (lane & 15)) * LDK + b_kb[it] * 32 + (lane >> 4) * 8;
    }
    const int kc = (tid % CPR) * 8;          // same for every chunk of this thread: NT % CPR == 0
    const bool pointwise = (p.KH * p.KW == 1);

    const int kt_begin = blockIdx.y * p.kt_per;
    const int kt_end = min(p.KT, kt_begin + p.kt_per);
    // K tiles are loaded strictly in order, so the thread keeps the position of its next 8 k, k = (kh, kw, ci),
    // and advances it by BK per tile without dividing.  Tiles at or beyond the end of the slice load zeros
    // (k >= k_lim), which keeps the K loops below free of branches.
    const int k_lim = min(p.K, kt_end * BK);
    const int kb_lim = min(KB, kt_end * KBT);
    int kb_run = kt_begin * KBT;
    int k_run = kt_begin * BK + kc;
    int kh_run = 0, kw_run = 0, ci_run = k_run;
    if (!pointwise) {
        const int tap = k_run / p.Cin;
        ci_run = k_run - tap * p.Cin;
        kh_run = tap / p.KW;
        kw_run = tap - kh_run * p.KW;
    }
    // state of the specialised forms: everything that moves along K is uniform over the workgroup
    int kt_run = kt_begin;                               // tile about to be loaded
    unsigned a_soff = (unsigned)kt_begin * BK * 2u;      // A_MATRIX: byte offset of that tile in a row of the operand
    unsigned b_soff = (unsigned)kt_begin * KBT * 1024u;  // byte offset of that tile's first k block in a row block of the weights
    int u_kh = 0, u_kw = 0, u_ci = kt_begin * BK;        // A_UNIFORM: window tap and first channel of that tile
    if (AMODE == A_UNIFORM) {
        const int tap = u_ci / p.Cin;
        u_ci -= tap * p.Cin;
        u_kh = tap / p.KW;
        u_kw = tap - u_kh * p.KW;
    }
    unsigned a_voff[A_IT], b_voff[B_IT];                 // constant per-thread offsets of the specialised forms
#pragma unroll
    for (int it = 0; it < A_IT; ++it) a_voff[it] = AMODE == A_MATRIX ? (a_ok[it] ? a_off0[it] + (unsigned)kc * 2u : OOB) : a_off0[it] + (unsigned)kc * 2u;
#pragma unroll
    for (int it = 0; it < B_IT; ++it) b_voff[it] = b_ok[it] ? b_base[it] + (unsigned)b_kb[it] * 1024u : OOB;
    // (written with & and selects rather than && and if: one basic block, so that the scheduler may spread these
    // instructions between matrix instructions)
    auto load_next = [&](uint4 (&ra)[A_IT], uint4 (&rb)[B_IT]) {
        if constexpr (AMODE == A_MATRIX) {
            const bool live = kt_run < kt_end;
#pragma unroll
            for (int it = 0; it < A_IT; ++it) {
                const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rx, live ? a_voff[it] : OOB, (int)a_soff, 0);
                ra[it] = make_uint4(v.x, v.y, v.z, v.w);
            }
#pragma unroll
            for (int it = 0; it < (BDIR ? 0 : B_IT); ++it) {
                const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rw, live ? b_voff[it] : OOB, (int)b_soff, 0);
                rb[it] = make_uint4(v.x, v.y, v.z, v.w);
            }
            ++kt_run;
            a_soff += BK * 2u;
            b_soff += KBT * 1024u;
            return;
        } else if constexpr (AMODE == A_UNIFORM) {
            const bool live = kt_run < kt_end;
            const unsigned tap_off = (unsigned)((u_kh * p.W + u_kw) * p.ldx + u_ci) * 2u;      // scalar
#pragma unroll
            for (int it = 0; it < A_IT; ++it) {
                const int ok = (int)a_ok[it] & (int)live & (int)((unsigned)(a_ih0[it] + u_kh) < (unsigned)p.H) &
                               (int)((unsigned)(a_iw0[it] + u_kw) < (unsigned)p.W);
                const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? a_voff[it] + tap_off : OOB, 0, 0);
                ra[it] = make_uint4(v.x, v.y, v.z, v.w);
            }
#pragma unroll
            for (int it = 0; it < (BDIR ? 0 : B_IT); ++it) {
                const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rw, live ? b_voff[it] : OOB, (int)b_soff, 0);
                rb[it] = make_uint4(v.x, v.y, v.z, v.w);
            }
            ++kt_run;
            b_soff += KBT * 1024u;
            u_ci += BK;
            if (u_ci >= p.Cin) {
                u_ci = 0;
                if (++u_kw == p.KW) { u_kw = 0; ++u_kh; }
            }
            return;
        }
        const int k_ok = k_run < k_lim;
        const unsigned tap_off = (unsigned)((kh_run * p.W + kw_run) * p.ldx + ci_run) * 2u;
#pragma unroll
        for (int it = 0; it < A_IT; ++it) {
            const int ok = (int)a_ok[it] & k_ok & (int)((unsigned)(a_ih0[it] + kh_run) < (unsigned)p.H) &
                           (int)((unsigned)(a_iw0[it] + kw_run) < (unsigned)p.W);
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? a_off0[it] + tap_off : OOB, 0, 0);
            ra[it] = make_uint4(v.x, v.y, v.z, v.w);
        }
#pragma unroll
        for (int it = 0; it < (BDIR ? 0 : B_IT); ++it) {
            const int kb = kb_run + b_kb[it];
            const int ok = (int)b_ok[it] & (int)(kb < kb_lim);
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rw, ok ? b_base[it] + (unsigned)kb * 1024u : OOB, 0, 0);
            rb[it] = make_uint4(v.x, v.y, v.z, v.w);
        }
        kb_run += KBT;
        k_run += BK;
        ci_run += BK;
        // Cin >= 8, so BK / 8 turns always suffice.  For a 1x1 window Cin == K and a wrap happens only beyond K,
        // where k_ok is false whatever the tap says.
#pragma unroll
        for (int u = 0; u < BK / 8; ++u) {
            const int wrap = ci_run >= p.Cin;
            ci_run -= wrap ? p.Cin : 0;
            kw_run += wrap;
            const int wrap2 = kw_run == p.KW;
            kw_run = wrap2 ? 0 : kw_run;
            kh_run += wrap2;
        }
    };
    auto store_tile = [&](int slot, const uint4 (&ra)[A_IT], const uint4 (&rb)[B_IT]) {
#pragma unroll
        for (int it = 0; it < A_IT; ++it) {
            const int c = tid + it * NT;
            if (A_CH % NT == 0 || c < A_CH) *reinterpret_cast<uint4 *>(&sA0[slot * BM * LDK + (c / CPR) * LDK + kc]) = ra[it];
        }
#pragma unroll
        for (int it = 0; it < (BDIR ? 0 : B_IT); ++it) {
            const int c = tid + it * NT;
            if (B_CH % NT == 0 || c < B_CH) *reinterpret_cast<uint4 *>(&sB0[slot * BN * LDK + b_lds[it]]) = rb[it];
        }
    };

    f32x4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int frag_row = lane & 15, frag_k = (lane >> 4) * 8;

    // RS register sets: set (t - kt_begin) % RS carries K step t, so RS steps of loads are in flight
    uint4 ra[RS][A_IT], rb[RS][B_IT];
#pragma unroll
    for (int r = 0; r < RS; ++r) load_next(ra[r], rb[r]);

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
    // The loop body is branch-free: steps at or beyond kt_end load zeros (k >= k_lim in load_next's terms is
    // forced by passing KT) and multiply them, which costs at most RS-1 idle steps at the end of a slice
    // and lets the compiler wait for exactly one step's loads at a time.
    if constexpr (BDIR) {
        // The ping-pong schedule below with the weights kept out of LDS.  Counters and a micro-benchmark put the LDS pipe,
        // not the matrix pipe, at the limit of the all-LDS form: a 16-byte-per-lane LDS read costs about 7 cycles of the
        // pipe and a write about 14, which for the 256 x 256 x 32 step adds up to 8 wavefronts x (12 reads + 4 writes) =
        // 1170 cycles against 1024 cycles of matrix instructions (192 x 128 x 64: 1500 against 770).  The weights are stored
        // in the order the matrix instruction consumes them (1 KB per 16 x 32 block, lane l owning bytes 16 l .. 16 l + 15),
        // so a wavefront can fetch its own fragments with one contiguous 1 KB load per block straight into the registers
        // the instruction reads: no LDS write and no LDS read for this operand, a third fewer LDS reads and half the LDS
        // writes per step.  The two wavefronts that share a column of the tile (wm = 0, 1) fetch the same blocks half a
        // step apart; the second fetch hits the compute unit's vector cache.
        // Fragments of step t+1 are requested in the matrix half-step of step t into the other half of fbq and are first
        // read one whole step later; the loads of the im2col tile t+RS+1 are issued after them, so that the in-order load
        // counter lets the matrix instructions start while those are still in flight.
        static_assert(WM * WN == 8, "ping-pong schedule: 8 wavefronts in two groups");
        constexpr int TK = BK / 32;
        const bool late = wave >= 4;
        unsigned fb_voff[TN];                    // this lane's 16 bytes in k block 0 of fragment j's row block
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int nb = ((n_base + wn * (BN / WN)) >> 4) + j;
            fb_voff[j] = nb < NB ? ((unsigned)nb * (unsigned)KB * 64u + (unsigned)lane) * 16u : OOB;
        }
        int fb_kb = kt_begin * KBT;              // first k block of the step whose fragments are requested next (uniform)
        uint4 fa[TK][TM], fbq[2][TK][TN];
        auto load_frags_b = [&](uint4 (&dst)[TK][TN]) {
#pragma unroll
            for (int ks = 0; ks < TK; ++ks) {
                const bool live = fb_kb + ks < kb_lim;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rw, live ? fb_voff[j] : OOB, (fb_kb + ks) * 1024, 0);
                    dst[ks][j] = make_uint4(v.x, v.y, v.z, v.w);
                }
            }
            fb_kb += KBT;
        };
        auto read_frags_a = [&](int slot) {
#pragma unroll
            for (int ks = 0; ks < TK; ++ks)
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    fa[ks][i] = *reinterpret_cast<const uint4 *>(&sA0[slot * BM * LDK + (wm * (BM / WM) + i * 16 + frag_row) * LDK + ks * 32 + frag_k]);
        };
        load_frags_b(fbq[0]);
        store_tile(0, ra[0], rb[0]);
        load_next(ra[0], rb[0]);
        __syncthreads();
        if (late) __syncthreads();
        for (int kt = kt_begin; kt < kt_end; kt += RS) {
#pragma unroll
            for (int r = 0; r < RS; ++r) {
                if (RS > 2 && kt + r >= kt_end) break;
                read_frags_a(r & 1);
                store_tile((r + 1) & 1, ra[(r + 1) % RS], rb[(r + 1) % RS]);
                __syncthreads();
                __builtin_amdgcn_s_setprio(1);
                load_frags_b(fbq[(r + 1) & 1]);
                load_next(ra[(r + 1) % RS], rb[(r + 1) % RS]);
#pragma unroll
                for (int ks = 0; ks < TK; ++ks)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j) acc[i][j] = Mma<T>::run(fbq[r & 1][ks][j], fa[ks][i], acc[i][j]);
                __builtin_amdgcn_s_setprio(0);
                __syncthreads();
            }
        }
        if (!late) __syncthreads();
    } else if constexpr (LOOP == LOOP_PINGPONG) {
        // Two groups of wavefronts, half a step apart.  Wavefronts w and w + 4 share a SIMD, and WN == 4 puts
        // them in different groups (group = wave / 4 = wm).  Time is cut into phases by workgroup barriers; in
        // every phase one group runs its memory half-step (fragments of step t from LDS into registers, tile
        // t+1 from registers into LDS) while the other issues the global loads of tile t+RS+1 and runs the MFMAs of its
        // previous half-step, so the matrix pipe and the LDS pipe of each SIMD are busy at the same time
        // instead of taking turns.  Group 1 starts one phase late and group 0 ends one phase late: both pass
        //   1 + (1 or 0) + 2 * steps + (0 or 1)
        // barriers, and the trip count is the same for every wavefront of a workgroup.
        // LDS hazards: slot s = (t+1)%2 is written in the memory half-steps of step t (phases 2t, 2t+1); its
        // previous content (tile t-1) was last read in phase 2t-1, and it is first read in phase 2t+2.
        static_assert(LOOP != LOOP_PINGPONG || (WM == 2 && WN == 4), "ping-pong schedule: 8 wavefronts in two groups");
        // Register stages: set r carries the tiles t with (t - kt_begin) % RS == r, so RS - 1 tiles are on their way
        // from memory while one is being moved to LDS.  What a step costs here is set by the bytes in flight, not by
        // the matrix pipe: with operands coming from HBM (weights of a large model are never cache-resident) a load
        // takes well over a microsecond under load, and two stages of a 192 x 128 x 64 step (80 KB per compute unit)
        // cover about half of that.  RS is even (the LDS slot of a stage is r & 1).
        constexpr int TK = BK / 32;              // matrix instructions along K per step and 16x16 block
        const bool late = wm != 0;
        uint4 fa[TK][TM], fb[TK][TN];
        auto read_frags = [&](int slot) {
#pragma unroll
            for (int ks = 0; ks < TK; ++ks) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    fb[ks][j] = *reinterpret_cast<const uint4 *>(&sB0[slot * BN * LDK + (wn * (BN / WN) + j * 16 + frag_row) * LDK + ks * 32 + frag_k]);
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    fa[ks][i] = *reinterpret_cast<const uint4 *>(&sA0[slot * BM * LDK + (wm * (BM / WM) + i * 16 + frag_row) * LDK + ks * 32 + frag_k]);
            }
        };
        // the loads of a later tile are issued from inside the MFMA half-step (their address arithmetic fills
        // issue slots between matrix instructions), which keeps the memory half-step down to LDS traffic
        auto mma = [&](uint4 (&na)[A_IT], uint4 (&nb)[B_IT]) {
            __builtin_amdgcn_s_setprio(1);
            load_next(na, nb);
#pragma unroll
            for (int ks = 0; ks < TK; ++ks)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) acc[i][j] = Mma<T>::run(fb[ks][j], fa[ks][i], acc[i][j]);
            __builtin_amdgcn_s_setprio(0);
        };
        store_tile(0, ra[0], rb[0]);
        load_next(ra[0], rb[0]);
        __syncthreads();
        if (late) __syncthreads();
        for (int kt = kt_begin; kt < kt_end; kt += RS) {
#pragma unroll
            for (int r = 0; r < RS; ++r) {
                // the trip count is the same for every wavefront of the workgroup (kt_end is uniform), so the
                // barriers stay matched when the last round is cut short
                if (RS > 2 && kt + r >= kt_end) break;
                read_frags(r & 1);
                store_tile((r + 1) & 1, ra[(r + 1) % RS], rb[(r + 1) % RS]);
                __syncthreads();
                mma(ra[(r + 1) % RS], rb[(r + 1) % RS]);
                __syncthreads();
            }
        }
        if (!late) __syncthreads();
    } else {
        for (int kt = kt_begin; kt < kt_end; kt += RS) {
#pragma unroll
            for (int r = 0; r < RS; ++r) {
                store_tile(r & 1, ra[r], rb[r]);
                __syncthreads();
                load_next(ra[r], rb[r]);
                compute(r & 1);
            }
        }
    }

    tile_epilogue<T, BM, BN, WM, WN, TM, TN>(p, acc, smem, m_base, n_base, blockIdx.y);
}


// Ping-pong tiles (8 wavefronts): X(variant id, BM, BN, BK, register stages, K-loop schedule).  Each is compiled in a
// translation unit of its own (k_gemm_pp.hip with ECLIP_PP_ID set), which exports launch_pp<ID> and init_pp<ID>.
// Ids 3 and 4 keep both operands in LDS (the 256 x 256 form is still the fastest on very large problems, where many
// workgroups contend for the vector cache); 5..14 fetch the weights straight into registers.
#define ECLIP_PP_TILES(X)                                                                                                   \
    X(3, 256, 256, 32, 2, LOOP_PINGPONG) X(4, 128, 256, 64, 2, LOOP_PINGPONG)                                               \
    X(5, 256, 256, 32, 2, LOOP_PP_BDIRECT) X(6, 128, 256, 64, 2, LOOP_PP_BDIRECT) X(7, 192, 128, 32, 2, LOOP_PP_BDIRECT)    \
    X(8, 192, 128, 64, 2, LOOP_PP_BDIRECT) X(9, 128, 128, 64, 2, LOOP_PP_BDIRECT) X(10, 256, 128, 32, 2, LOOP_PP_BDIRECT)   \
    X(11, 192, 256, 32, 2, LOOP_PP_BDIRECT) X(12, 256, 192, 32, 2, LOOP_PP_BDIRECT) X(13, 64, 128, 64, 2, LOOP_PP_BDIRECT)  \
    X(14, 128, 64, 64, 2, LOOP_PP_BDIRECT) X(15, 96, 64, 64, 2, LOOP_PP_BDIRECT) X(16, 96, 192, 64, 2, LOOP_PP_BDIRECT)

struct PPTile { int id, bm, bn, bk, rs, loop; };
constexpr PPTile kPPTiles[] = {
#define X(ID, BM, BN, BK, RS, LP) {ID, BM, BN, BK, RS, LP},
    ECLIP_PP_TILES(X)
#undef X
};
constexpr PPTile pp_tile(int id)
{
    for (const PPTile &t : kPPTiles)
        if (t.id == id) return t;
    return PPTile{-1, 0, 0, 0, 0, 0};
}

// LDS of a workgroup: the two-slot operand ring, or the epilogue's staging buffers when those are larger (8 wavefronts
// x 32 rows x (columns of a wavefront + 4) floats on the ping-pong tiles)
constexpr size_t lds_bytes(int bm, int bn, int bk, int pad = 8, bool weights_in_lds = true)
{
    const size_t ring = (size_t)2 * (bm + (weights_in_lds ? bn : 0)) * (bk + pad) * 2;
    const size_t stage = pad == 16 ? (size_t)8 * 32 * (bn / 4 + 4) * 4 : 0;
    return ring > stage ? ring : stage;
}

// Which addressing form a launch may take (see conv_gemm_kernel)
inline int gemm_amode(const GemmDev &d, int bk)
{
    if (d.nchw_c) return A_GENERAL;
    if (d.KH * d.KW == 1 && d.pad == 0 && d.K % bk == 0) return A_MATRIX;
    if (d.Cin % bk == 0) return A_UNIFORM;
    return A_GENERAL;
}

template <int ID> hipError_t launch_pp(const GemmDev &d, int dtype, dim3 grid, hipStream_t s);
template <int ID> hipError_t init_pp();

}  // namespace eclip
