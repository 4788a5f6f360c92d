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
        static_assert(TM % 2 == 0, "32 rows per pass");
        constexpr int COLS = TN * 16, SP = COLS + 4;          // row pitch in floats: the 4-float pad spreads the banks
        constexpr int LPR = COLS / 8, RPP = 64 / LPR;          // lanes per row, rows per pass (lanes beyond RPP * LPR idle)
        constexpr int PASSES = (32 + RPP - 1) / RPP;
        __syncthreads();
        float *stage = reinterpret_cast<float *>(smem) + wave * (32 * SP);
        const int rr0 = lane / LPR, col8 = (lane % LPR) * 8;
        const int n = n_base + wn * (BN / WN) + col8;
        static_for<TM / 2>([&](auto hc) {
            constexpr int h = decltype(hc)::value;
            static_for<2>([&](auto ic) {
                constexpr int i2 = decltype(ic)::value;
                static_for<TN>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
                    const f32x4 a4 = acc[2 * h + i2][j];
                    *reinterpret_cast<float4 *>(&stage[(i2 * 16 + (lane & 15)) * SP + j * 16 + (lane >> 4) * 4]) = make_float4(a4[0], a4[1], a4[2], a4[3]);
                });
            });
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_s_waitcnt(0xc07f);              // lgkmcnt(0): this wavefront's LDS writes have landed
            auto pass = [&](int ps) {
                const int rr = ps * RPP + rr0;
                const int m = m_base + wm * (BM / WM) + h * 32 + rr;
                if (lane < RPP * LPR && rr < 32 && m < p.M && n < p.N) {
                    const float4 q0 = *reinterpret_cast<const float4 *>(&stage[rr * SP + col8]);
                    const float4 q1 = *reinterpret_cast<const float4 *>(&stage[rr * SP + col8 + 4]);
                    float o[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
                    if constexpr (N8) epilogue_store8<T, ACT>(p.bias, p.res, p.y, p.y32, p.N, m, n, o);
                    else epilogue_store8_ragged<T, ACT>(p.bias, p.res, p.y, p.y32, p.N, m, n, o);
                }
            };
            if constexpr (N8) {
#pragma unroll
                for (int ps = 0; ps < PASSES; ++ps) pass(ps);
            } else {
#pragma unroll 1
                for (int ps = 0; ps < PASSES; ++ps) pass(ps);
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
enum { LOOP_PLAIN = 0, LOOP_PINGPONG = 2 };

template <typename T, int BM, int BN, int BK, int WM, int WN, int RS, int LOOP = LOOP_PLAIN>
__global__ __launch_bounds__(WM * WN * 64) void conv_gemm_kernel(GemmDev p)
{
    constexpr int NT = WM * WN * 64;         // threads per workgroup: 4 wavefronts, 8 for the 256x256 tile
    static_assert(RS % 2 == 0, "register stages alternate between the two LDS slots");
    // row pitch in elements.  Measured with a ds_read_b128 / ds_write_b128 micro-benchmark: with 64-byte rows a
    // pitch of 96 bytes makes the fragment reads (16 rows x 4 chunks per instruction) conflict-free, 80 bytes
    // costs them about 20 %.
    constexpr int LDK = (LOOP == LOOP_PINGPONG) ? BK + 16 : BK + 8;
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
        a_off0[it] = ((unsigned)b * (unsigned)(p.H * p.W) + (unsigned)(a_ih0[it] * p.W + a_iw0[it])) * (unsigned)p.Cin * 2u;
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
    // (written with & and selects rather than && and if: one basic block, so that the scheduler may spread these
    // instructions between matrix instructions)
    auto load_next = [&](uint4 (&ra)[A_IT], uint4 (&rb)[B_IT]) {
        const int k_ok = k_run < k_lim;
        const unsigned tap_off = (unsigned)((kh_run * p.W + kw_run) * p.Cin + ci_run) * 2u;
#pragma unroll
        for (int it = 0; it < A_IT; ++it) {
            const int ok = (int)a_ok[it] & k_ok & (int)((unsigned)(a_ih0[it] + kh_run) < (unsigned)p.H) &
                           (int)((unsigned)(a_iw0[it] + kw_run) < (unsigned)p.W);
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? a_off0[it] + tap_off : OOB, 0, 0);
            ra[it] = make_uint4(v.x, v.y, v.z, v.w);
        }
#pragma unroll
        for (int it = 0; it < B_IT; ++it) {
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
        for (int it = 0; it < B_IT; ++it) {
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
    if constexpr (LOOP == LOOP_PINGPONG) {
        // Two groups of wavefronts, half a step apart.  Wavefronts w and w + 4 share a SIMD, and WN == 4 puts
        // them in different groups (group = wave / 4 = wm).  Time is cut into phases by workgroup barriers; in
        // every phase one group runs its memory half-step (fragments of step t from LDS into registers, tile
        // t+1 from registers into LDS) while the other issues the global loads of tile t+3 and runs the MFMAs of its
        // previous half-step, so the matrix pipe and the LDS pipe of each SIMD are busy at the same time
        // instead of taking turns.  Group 1 starts one phase late and group 0 ends one phase late: both pass
        //   1 + (1 or 0) + 2 * steps + (0 or 1)
        // barriers, and the trip count is the same for every wavefront of a workgroup.
        // LDS hazards: slot s = (t+1)%2 is written in the memory half-steps of step t (phases 2t, 2t+1); its
        // previous content (tile t-1) was last read in phase 2t-1, and it is first read in phase 2t+2.
        static_assert(LOOP != LOOP_PINGPONG || (RS == 2 && WM == 2 && WN == 4), "ping-pong schedule: 8 wavefronts, two register sets");
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
        for (int kt = kt_begin; kt < kt_end; kt += 2) {
            read_frags(0);
            store_tile(1, ra[1], rb[1]);
            __syncthreads();
            mma(ra[1], rb[1]);
            __syncthreads();
            read_frags(1);
            store_tile(0, ra[0], rb[0]);
            __syncthreads();
            mma(ra[0], rb[0]);
            __syncthreads();
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
#define EPI(A) epilogue_store<T, A>(bias, res, y, y32, M, N, m, n, s, vec ? 4 : 1)
    ECLIP_ACT_SWITCH(act, EPI)
#undef EPI
}

struct Variant { int bm, bn, bk; };
constexpr Variant kVariants[CONV_GEMM_VARIANTS] = {{128, 128, 32}, {64, 64, 64}, {32, 64, 64}, {256, 256, 32}, {128, 256, 64},
                                                   {192, 128, 32}, {192, 128, 64}, {128, 128, 64}, {256, 128, 32}, {192, 256, 32},
                                                   {256, 192, 32}, {64, 128, 64}, {128, 64, 64}};

// LDS of a workgroup: the two-slot operand ring, or the epilogue's staging buffers when those are larger (8 wavefronts
// x 32 rows x (columns of a wavefront + 4) floats on the ping-pong tiles)
constexpr size_t lds_bytes(int bm, int bn, int bk, int pad = 8)
{
    const size_t ring = (size_t)2 * (bm + bn) * (bk + pad) * 2;
    const size_t stage = pad == 16 ? (size_t)8 * 32 * (bn / 4 + 4) * 4 : 0;
    return ring > stage ? ring : stage;
}

template <typename T>
hipError_t launch_t(const GemmDev &d, const GemmPlan &pl, hipStream_t s)
{
    const dim3 grid((unsigned)pl.tiles, (unsigned)pl.splits);
    switch (pl.variant) {
    case 0: hipLaunchKernelGGL((conv_gemm_kernel<T, 128, 128, 32, 2, 2, 2>), grid, dim3(256), lds_bytes(128, 128, 32), s, d); break;
    case 1: hipLaunchKernelGGL((conv_gemm_kernel<T, 64, 64, 64, 2, 2, 4>), grid, dim3(256), lds_bytes(64, 64, 64), s, d); break;
    case 2: hipLaunchKernelGGL((conv_gemm_kernel<T, 32, 64, 64, 1, 4, 4>), grid, dim3(256), lds_bytes(32, 64, 64), s, d); break;
#define PP(BM, BN, BK) hipLaunchKernelGGL((conv_gemm_kernel<T, BM, BN, BK, 2, 4, 2, LOOP_PINGPONG>), grid, dim3(512), lds_bytes(BM, BN, BK, 16), s, d)
    case 3: PP(256, 256, 32); break;
    case 4: PP(128, 256, 64); break;
    case 5: PP(192, 128, 32); break;
    case 6: PP(192, 128, 64); break;
    case 7: PP(128, 128, 64); break;
    case 8: PP(256, 128, 32); break;
    case 9: PP(192, 256, 32); break;
    case 10: PP(256, 192, 32); break;
    case 11: PP(64, 128, 64); break;
    default: PP(128, 64, 64); break;
#undef PP
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
    hipError_t e;
#define SET(T, BM, BN, BK)                                                                                                   \
    if ((e = hipFuncSetAttribute((const void *)conv_gemm_kernel<T, BM, BN, BK, 2, 4, 2, LOOP_PINGPONG>,                      \
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes(BM, BN, BK, 16))) != hipSuccess) \
        return e;
#define SET2(BM, BN, BK) SET(bf16_t, BM, BN, BK) SET(f16_t, BM, BN, BK)
    SET2(256, 256, 32) SET2(128, 256, 64) SET2(192, 128, 32) SET2(192, 128, 64) SET2(128, 128, 64) SET2(256, 128, 32)
    SET2(192, 256, 32) SET2(256, 192, 32) SET2(64, 128, 64) SET2(128, 64, 64)
#undef SET2
#undef SET
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
    // LDS-tiled kernel, optionally with K cut in two (second launch: its cost plus the traffic of the partial sums).
    // A tile costs `shared` us per K step when workgroups share a compute unit and `alone` when it has one to itself.
    struct { int variant; double shared, alone, fixed; } lds[4] = {{0, 0.3613, 0.6385, 0.02038}, {1, 0.3664, 1.171, 0.1703}, {3, 0.7721, 0.7721, 0.554},
                                                                   {4, 1.157, 1.157, 2.62}};
    for (const auto &c : lds) {
        int bm, bn, bk;
        conv_gemm_tile(c.variant, &bm, &bn, &bk);
        const long KT = cdiv(K, bk);
        for (long sp = 1; sp <= (c.variant == 3 ? 1 : 2); ++sp) {
            if (sp > 1 && (K < 512 || (size_t)(sp * M * N) > ws_floats)) continue;
            const long wgs = tiles(c.variant) * sp, per_cu = cdiv(wgs, n_cu);
            double cost = c.fixed + (double)cdiv(KT, sp) * (per_cu == 1 ? c.alone : (double)per_cu * c.shared);
            if (sp == 1 && c.variant == 1) cost *= 1.35;          // residuals of the fit, as for the other kernel
            if (sp == 1 && c.variant == 0) cost -= 0.1;
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
    d.x_bytes = (unsigned)((size_t)a.B * a.H * a.W * (a.nchw_c ? a.nchw_c : a.Cin) * 2);
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
    if (n_launched) *n_launched += 1;
    return launch_conv_wsk_pair(make_dev(a0, p0), p0.tiles, make_dev(a1, p1), p1.tiles, a0.dtype, p0.variant, p0.nw, s);
}

}  // namespace eclip
