// Fused multi-head attention for short sequences (S <= 512, head size 32 or 64):
//   out[b, s, h*d + j] = sum_t softmax_t(q_s . k_t / sqrt(d)) v_t[j]
// with q, k, v read from one [B][S][3*Hd] tensor ([q | k | v], head-major).
//
// One workgroup of NW wavefronts handles NW*16 query rows of one (batch, head).  Per wavefront:
//   1. scores: for every block of 16 keys, D[key][query] = K_blk (16 x d) . Q^T (d x 16) with
//      v_mfma_f32_16x16x32 (d/32 instructions); a lane then holds, for its query (lane & 15), the 4
//      keys 4*(lane>>4)..+3 of every key block -- the whole score row stays in registers;
//   2. softmax over keys: in-lane over blocks and the 4 values, then across the 4 lane groups that
//      share a query (xor-shuffles by 16 and 32); fp32 throughout;
//   3. out^T = V^T . P^T: the contraction index of one MFMA covers two key blocks; the lane's own 8
//      probabilities (4 per block) are already the column operand it must supply, and V^T is read from
//      an LDS copy transposed on load so that the matching 4 keys are 8 contiguous bytes.
// The unnormalised probabilities (exp of score minus row maximum, in (0, 1]) are rounded to the 16-bit type for the
// second product and the division by the row sum is applied to the outputs; scores are never stored.
// The key fragments come straight from global memory for up to 256 keys (all loads of the workgroup in flight at
// once: attention_kernel); beyond that the keys too are staged in LDS by the whole workgroup with row-contiguous loads
// and shared by its wavefronts (fetched per wavefront in fragment order, 48 dependent round trips made S = 384 take
// 45 us), one chunk of keys at a time (attention_chunk_kernel).
#include "device_common.h"
#include "kernels.h"

namespace eclip {

namespace {

template <typename T> struct MmaA;
template <> struct MmaA<bf16_t> {
    __device__ static __forceinline__ f32x4 run(uint4 a, uint4 b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct MmaA<f16_t> {
    __device__ static __forceinline__ f32x4 run(uint4 a, uint4 b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};

struct AttnDev {
    const uint16_t *qkv;
    uint16_t *y;
    float *y32;
    int B, S, Hd, heads, Sp, ldv;   // Sp = S rounded up to 32; ldv = LDS pitch of V^T in elements
    int ck, nchunks;                // chunked kernel: keys per chunk (a multiple of 32) and number of chunks
    float scale;
};

// KB = number of 16-key blocks held in registers (Sp / 16 <= KB <= 16)
template <typename T, int D, int KB, int NW>
__global__ __launch_bounds__(NW * 64) void attention_kernel(AttnDev p)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t vt[];    // [D][ldv]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int qblocks = (p.S + NW * 16 - 1) / (NW * 16);
    const int qb = blockIdx.x % qblocks;
    const int bh = blockIdx.x / qblocks;
    const int h = bh % p.heads, b = bh / p.heads;
    const long row0 = (long)b * p.S;
    const int ld = 3 * p.Hd;
    const uint16_t *qp = p.qkv + h * D;
    const uint16_t *kp = p.qkv + p.Hd + h * D;
    const uint16_t *vp = p.qkv + 2 * p.Hd + h * D;

    const int q_row = qb * NW * 16 + wave * 16 + (lane & 15);      // this lane's query
    const int g = lane >> 4;                                        // lane group: contraction chunk / key quad
    const bool q_ok = q_row < p.S;

    // ---- Q fragments (column operand): 8 consecutive head dims per lane and 32-wide K step
    uint4 qf[D / 32];
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks) {
        qf[ks] = make_uint4(0, 0, 0, 0);
        if (q_ok) qf[ks] = *reinterpret_cast<const uint4 *>(qp + (row0 + q_row) * ld + ks * 32 + g * 8);
    }

    // The K fragments too are fetched before the V^T fill, so that all global loads of the workgroup are in flight
    // together (one memory round trip instead of three).
    uint4 kfr[KB][D / 32];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int ks = 0; ks < D / 32; ++ks) {
            const int key = kb * 16 + (lane & 15);
            kfr[kb][ks] = make_uint4(0, 0, 0, 0);
            if (key < p.S) kfr[kb][ks] = *reinterpret_cast<const uint4 *>(kp + (row0 + key) * ld + ks * 32 + g * 8);
        }

    // ---- V^T into LDS.  A thread loads 8 consecutive head dims of 4 consecutive keys (four 16-byte loads), turns the
    // 4 x 8 block in registers and writes, for each of the 8 head dims, its 4 keys as one 8-byte word; consecutive
    // lanes take consecutive key quads, so every store instruction of a wavefront writes 512 contiguous bytes.
    auto load_v = [&](int c, uint32_t (&w)[4][4]) {
        const int kq = c % (p.Sp / 4), j0 = (c / (p.Sp / 4)) * 8, key0 = kq * 4;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            uint4 q = make_uint4(0, 0, 0, 0);
            if (c < (p.Sp / 4) * (D / 8) && key0 + t < p.S) q = *reinterpret_cast<const uint4 *>(vp + (row0 + key0 + t) * ld + j0);
            w[t][0] = q.x; w[t][1] = q.y; w[t][2] = q.z; w[t][3] = q.w;
        }
    };
    auto store_vt = [&](int c, const uint32_t (&w)[4][4]) {
        if (c >= (p.Sp / 4) * (D / 8)) return;
        const int kq = c % (p.Sp / 4), j0 = (c / (p.Sp / 4)) * 8, key0 = kq * 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint2 lo = make_uint2((w[0][i] & 0xffffu) | (w[1][i] << 16), (w[2][i] & 0xffffu) | (w[3][i] << 16));
            const uint2 hi = make_uint2((w[0][i] >> 16) | (w[1][i] & 0xffff0000u), (w[2][i] >> 16) | (w[3][i] & 0xffff0000u));
            *reinterpret_cast<uint2 *>(&vt[(j0 + 2 * i) * p.ldv + key0]) = lo;
            *reinterpret_cast<uint2 *>(&vt[(j0 + 2 * i + 1) * p.ldv + key0]) = hi;
        }
    };
    for (int c = tid; c < (p.Sp / 4) * (D / 8); c += NW * 64) {
        uint32_t w[4][4];
        load_v(c, w);
        store_vt(c, w);
    }
    __syncthreads();

    // ---- scores
    f32x4 sc[KB];
    const int nkb = p.Sp / 16;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        sc[kb] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (kb < nkb) {
#pragma unroll
            for (int ks = 0; ks < D / 32; ++ks) sc[kb] = MmaA<T>::run(kfr[kb][ks], qf[ks], sc[kb]);
        }
    }

    // ---- softmax over keys (lane holds keys kb*16 + 4*g + r).  The vector ALU is what this kernel waits for (96 scores
    // per lane at 384 keys), so the row is touched as few times as possible: the maximum is taken over the raw scores
    // (the scale is positive), exp((s - max) * scale) is one fused multiply-add and one exp2, padded keys are masked only
    // in the blocks that contain any, and the division by the sum is applied to the 16 outputs instead of the scores.
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
        if (kb < nkb) {
            if ((kb + 1) * 16 > p.S) {           // wavefront-uniform: only the last blocks hold padded keys
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (kb * 16 + 4 * g + r >= p.S) sc[kb][r] = -INFINITY;
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) mx = fmaxf(mx, sc[kb][r]);
        }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float c2 = p.scale * 1.4426950408889634f, off2 = -mx * c2;
    float sum = 0.0f;

    // ---- out^T[j][query] = sum_key V^T[j][key] * P[query][key], the exponentials taken pair of key blocks by pair of key
    // blocks so that vector-ALU work and the LDS reads and matrix instructions of the product alternate
    f32x4 o[D / 16];
#pragma unroll
    for (int jb = 0; jb < D / 16; ++jb) o[jb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kp2 = 0; kp2 < KB / 2; ++kp2) {
        if (2 * kp2 < nkb) {
#pragma unroll
            for (int kb = 2 * kp2; kb < 2 * kp2 + 2; ++kb)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float e = __builtin_amdgcn_exp2f(fmaf(sc[kb][r], c2, off2));      // exp2(-inf) = 0 for padded keys
                    sc[kb][r] = e;
                    sum += e;
                }
            // contraction slot e of lane group g  <->  key (2*kp2 + e/4)*16 + 4*g + e%4
            uint4 pf;
            pf.x = Cvt<T>::pack2(sc[2 * kp2][0], sc[2 * kp2][1]);
            pf.y = Cvt<T>::pack2(sc[2 * kp2][2], sc[2 * kp2][3]);
            pf.z = Cvt<T>::pack2(sc[2 * kp2 + 1][0], sc[2 * kp2 + 1][1]);
            pf.w = Cvt<T>::pack2(sc[2 * kp2 + 1][2], sc[2 * kp2 + 1][3]);
#pragma unroll
            for (int jb = 0; jb < D / 16; ++jb) {
                const uint16_t *vr = vt + (jb * 16 + (lane & 15)) * p.ldv + 4 * g;
                const uint2 lo = *reinterpret_cast<const uint2 *>(vr + (2 * kp2) * 16);
                const uint2 hi = *reinterpret_cast<const uint2 *>(vr + (2 * kp2 + 1) * 16);
                o[jb] = MmaA<T>::run(make_uint4(lo.x, lo.y, hi.x, hi.y), pf, o[jb]);
            }
        }
    }

    sum += __shfl_xor(sum, 16, 64);
    sum += __shfl_xor(sum, 32, 64);
    const float inv = 1.0f / sum;
    // lane holds head dims jb*16 + 4*g .. +3 of its query
#pragma unroll
    for (int jb = 0; jb < D / 16; ++jb)
#pragma unroll
        for (int r = 0; r < 4; ++r) o[jb][r] *= inv;
    if (q_ok) {
        const long off = (row0 + q_row) * p.Hd + h * D + 4 * g;
#pragma unroll
        for (int jb = 0; jb < D / 16; ++jb) {
            if (p.y32) {
                *reinterpret_cast<float4 *>(p.y32 + off + jb * 16) = make_float4(o[jb][0], o[jb][1], o[jb][2], o[jb][3]);
            } else {
                uint2 q;
                q.x = Cvt<T>::pack2(o[jb][0], o[jb][1]);
                q.y = Cvt<T>::pack2(o[jb][2], o[jb][3]);
                *reinterpret_cast<uint2 *>(p.y + off + jb * 16) = q;
            }
        }
    }
}

// More than 256 keys: the keys are taken in chunks of p.ck (two chunks for up to 512 keys) with a running maximum and
// sum, so that a workgroup stages only one chunk of K and V^T in LDS (53 KB at 384 keys and head size 64 instead of
// 105 KB) and holds only one chunk of scores in registers: two workgroups then share a CU, and one's loads, LDS fill
// and barriers overlap the other's arithmetic (holding the next chunk's loads in registers across the arithmetic would
// cost the second workgroup: 156 registers per lane against the 128 that sixteen wavefronts leave).  Between chunks the 16 outputs and the sum of a query are scaled by
// exp(old maximum - new maximum); everything else is as in attention_kernel.  KBC = 16-key blocks per chunk held in
// registers (p.ck / 16 <= KBC).
template <typename T, int D, int KBC, int NW>
__global__ __launch_bounds__(NW * 64, (NW == 8 && KBC <= 12) ? 4 : 2) void attention_chunk_kernel(AttnDev p)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t vt[];    // V^T chunk [D][ldv], then the key chunk [ck][D + 8]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int qblocks = (p.S + NW * 16 - 1) / (NW * 16);
    const int qb = blockIdx.x % qblocks;
    const int bh = blockIdx.x / qblocks;
    const int h = bh % p.heads, b = bh / p.heads;
    const long row0 = (long)b * p.S;
    const int ld = 3 * p.Hd;
    const uint16_t *qp = p.qkv + h * D;
    const uint16_t *kp = p.qkv + p.Hd + h * D;
    const uint16_t *vp = p.qkv + 2 * p.Hd + h * D;
    const int q_row = qb * NW * 16 + wave * 16 + (lane & 15);
    const int g = lane >> 4;
    const bool q_ok = q_row < p.S;
    const int ck = p.ck, nkb = ck / 16;

    uint4 qf[D / 32];
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks) {
        qf[ks] = make_uint4(0, 0, 0, 0);
        if (q_ok) qf[ks] = *reinterpret_cast<const uint4 *>(qp + (row0 + q_row) * ld + ks * 32 + g * 8);
    }

    constexpr int KP = D + 8, CPR = D / 8;
    constexpr int K_IT = (KBC * 16 * CPR + NW * 64 - 1) / (NW * 64);          // 16-byte key chunks per thread and chunk
    constexpr int V_IT = (KBC * 4 * CPR + NW * 64 - 1) / (NW * 64);           // 4-key x 8-dim V blocks per thread and chunk
    uint16_t *const kl = vt + D * p.ldv;
    const int vq = ck / 4;                                                    // key quads per chunk
    uint4 kq[K_IT];
    uint32_t vw[V_IT][4][4];
    // global -> registers: keys [key0, key0 + ck); rows beyond S read as zeros
    auto fetch = [&](int key0) {
#pragma unroll
        for (int it = 0; it < K_IT; ++it) {
            const int c = tid + it * NW * 64, key = c / CPR, j0 = (c % CPR) * 8;
            kq[it] = make_uint4(0, 0, 0, 0);
            if (key < ck && key0 + key < p.S) kq[it] = *reinterpret_cast<const uint4 *>(kp + (row0 + key0 + key) * ld + j0);
        }
#pragma unroll
        for (int it = 0; it < V_IT; ++it) {
            const int c = tid + it * NW * 64, k0 = (c % vq) * 4, j0 = (c / vq) * 8;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                uint4 q = make_uint4(0, 0, 0, 0);
                if (c < vq * CPR && key0 + k0 + t < p.S) q = *reinterpret_cast<const uint4 *>(vp + (row0 + key0 + k0 + t) * ld + j0);
                vw[it][t][0] = q.x; vw[it][t][1] = q.y; vw[it][t][2] = q.z; vw[it][t][3] = q.w;
            }
        }
    };
    // registers -> LDS: key rows as they are, V turned so that 4 keys of a head dim are one 8-byte word
    auto stash = [&]() {
#pragma unroll
        for (int it = 0; it < K_IT; ++it) {
            const int c = tid + it * NW * 64, key = c / CPR, j0 = (c % CPR) * 8;
            if (key < ck) *reinterpret_cast<uint4 *>(&kl[key * KP + j0]) = kq[it];
        }
#pragma unroll
        for (int it = 0; it < V_IT; ++it) {
            const int c = tid + it * NW * 64, k0 = (c % vq) * 4, j0 = (c / vq) * 8;
            if (c < vq * CPR) {
                const uint32_t(&w)[4][4] = vw[it];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint2 lo = make_uint2((w[0][i] & 0xffffu) | (w[1][i] << 16), (w[2][i] & 0xffffu) | (w[3][i] << 16));
                    const uint2 hi = make_uint2((w[0][i] >> 16) | (w[1][i] & 0xffff0000u), (w[2][i] >> 16) | (w[3][i] & 0xffff0000u));
                    *reinterpret_cast<uint2 *>(&vt[(j0 + 2 * i) * p.ldv + k0]) = lo;
                    *reinterpret_cast<uint2 *>(&vt[(j0 + 2 * i + 1) * p.ldv + k0]) = hi;
                }
            }
        }
    };

    f32x4 o[D / 16];
#pragma unroll
    for (int jb = 0; jb < D / 16; ++jb) o[jb] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, sum = 0.0f;
    const float c2 = p.scale * 1.4426950408889634f;
    for (int c = 0; c < p.nchunks; ++c) {
        const int key0 = c * ck;
        fetch(key0);
        if (c > 0) __syncthreads();                   // every wavefront is done reading the previous chunk
        stash();
        __syncthreads();

        f32x4 sc[KBC];
#pragma unroll
        for (int kb = 0; kb < KBC; ++kb) {
            sc[kb] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (kb < nkb) {
#pragma unroll
                for (int ks = 0; ks < D / 32; ++ks) {
                    const uint4 kf = *reinterpret_cast<const uint4 *>(&kl[(kb * 16 + (lane & 15)) * KP + ks * 32 + g * 8]);
                    sc[kb] = MmaA<T>::run(kf, qf[ks], sc[kb]);
                }
            }
        }
        float mc = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < KBC; ++kb)
            if (kb < nkb) {
                if (key0 + (kb + 1) * 16 > p.S) {     // wavefront-uniform: only the last blocks hold padded keys
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (key0 + kb * 16 + 4 * g + r >= p.S) sc[kb][r] = -INFINITY;
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) mc = fmaxf(mc, sc[kb][r]);
            }
        mc = fmaxf(mc, __shfl_xor(mc, 16, 64));
        mc = fmaxf(mc, __shfl_xor(mc, 32, 64));
        // every chunk holds at least one key below S (checked at launch), so the new maximum is finite; in the first
        // chunk the old one is -inf and the factor exp2(-inf) = 0 scales sums that are still zero
        const float m_new = fmaxf(m_run, mc);
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c2);
        m_run = m_new;
        const float off2 = -m_new * c2;
#pragma unroll
        for (int jb = 0; jb < D / 16; ++jb)
#pragma unroll
            for (int r = 0; r < 4; ++r) o[jb][r] *= alpha;

        // exponentials and P.V pair of key blocks by pair of key blocks, so that the vector ALU (8 exp2 per pair) and the
        // LDS reads and matrix instructions of the product alternate in every wavefront's instruction stream instead of
        // forming two long phases that all wavefronts of the workgroup enter together
        float part = 0.0f;
#pragma unroll
        for (int kp2 = 0; kp2 < KBC / 2; ++kp2) {
            if (2 * kp2 < nkb) {
#pragma unroll
                for (int kb = 2 * kp2; kb < 2 * kp2 + 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float e = __builtin_amdgcn_exp2f(fmaf(sc[kb][r], c2, off2));
                        sc[kb][r] = e;
                        part += e;
                    }
                uint4 pf;
                pf.x = Cvt<T>::pack2(sc[2 * kp2][0], sc[2 * kp2][1]);
                pf.y = Cvt<T>::pack2(sc[2 * kp2][2], sc[2 * kp2][3]);
                pf.z = Cvt<T>::pack2(sc[2 * kp2 + 1][0], sc[2 * kp2 + 1][1]);
                pf.w = Cvt<T>::pack2(sc[2 * kp2 + 1][2], sc[2 * kp2 + 1][3]);
#pragma unroll
                for (int jb = 0; jb < D / 16; ++jb) {
                    const uint16_t *vr = vt + (jb * 16 + (lane & 15)) * p.ldv + 4 * g;
                    const uint2 lo = *reinterpret_cast<const uint2 *>(vr + (2 * kp2) * 16);
                    const uint2 hi = *reinterpret_cast<const uint2 *>(vr + (2 * kp2 + 1) * 16);
                    o[jb] = MmaA<T>::run(make_uint4(lo.x, lo.y, hi.x, hi.y), pf, o[jb]);
                }
            }
        }
        sum = fmaf(sum, alpha, part);
    }
    sum += __shfl_xor(sum, 16, 64);
    sum += __shfl_xor(sum, 32, 64);
    const float inv = 1.0f / sum;
#pragma unroll
    for (int jb = 0; jb < D / 16; ++jb)
#pragma unroll
        for (int r = 0; r < 4; ++r) o[jb][r] *= inv;
    if (q_ok) {
        const long off = (row0 + q_row) * p.Hd + h * D + 4 * g;
#pragma unroll
        for (int jb = 0; jb < D / 16; ++jb) {
            if (p.y32) {
                *reinterpret_cast<float4 *>(p.y32 + off + jb * 16) = make_float4(o[jb][0], o[jb][1], o[jb][2], o[jb][3]);
            } else {
                uint2 q;
                q.x = Cvt<T>::pack2(o[jb][0], o[jb][1]);
                q.y = Cvt<T>::pack2(o[jb][2], o[jb][3]);
                *reinterpret_cast<uint2 *>(p.y + off + jb * 16) = q;
            }
        }
    }
}

inline int round_up(int a, int b) { return (a + b - 1) / b * b; }
// LDS row pitch of V^T in elements, keys + 4: a lane reads 8 bytes of row (lane & 15), and with the pitch an odd
// multiple of 8 bytes the 16 rows fall on 16 different pairs of banks (with keys + 8, the pitch a multiple of 16
// bytes, rows r and r + 8 share their banks: SQ_LDS_BANK_CONFLICT 2.9 per active LDS cycle, 1.1 with keys + 4, and
// 380 -> 348 us at 4096 (batch, head) pairs of 384 keys)
inline int ldv_of(int keys) { return keys + 4; }

template <typename T, int D, int NW>
hipError_t launch_d(const AttnDev &d, size_t lds, hipStream_t s)
{
    const int qblocks = (d.S + NW * 16 - 1) / (NW * 16);
    const dim3 grid((unsigned)(d.B * d.heads * qblocks)), block(NW * 64);
    const int nkb = d.Sp / 16;
    if (nkb <= 8) hipLaunchKernelGGL((attention_kernel<T, D, 8, NW>), grid, block, lds, s, d);
    else if (nkb <= 16) hipLaunchKernelGGL((attention_kernel<T, D, 16, NW>), grid, block, lds, s, d);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

template <typename T, int D, int NW>
hipError_t launch_chunked(const AttnDev &d, size_t lds, hipStream_t s)
{
    const int qblocks = (d.S + NW * 16 - 1) / (NW * 16);
    const dim3 grid((unsigned)(d.B * d.heads * qblocks)), block(NW * 64);
    if (d.ck % 32 != 0 || d.ck > 256 || d.nchunks * d.ck < d.Sp || (d.nchunks - 1) * d.ck >= d.S) return hipErrorInvalidValue;
    if (d.ck <= 192) hipLaunchKernelGGL((attention_chunk_kernel<T, D, 12, NW>), grid, block, lds, s, d);
    else hipLaunchKernelGGL((attention_chunk_kernel<T, D, 16, NW>), grid, block, lds, s, d);
    return hipGetLastError();
}

template <typename T, int D, int NW>
hipError_t set_attr()
{
    const int lim = 96 * 1024;               // 512 keys: chunks of 256, 34 KB of V^T + 37 KB of keys
    if constexpr (NW == 4 || NW == 8) {
        hipError_t e;
        if ((e = hipFuncSetAttribute((const void *)attention_chunk_kernel<T, D, 12, NW>, hipFuncAttributeMaxDynamicSharedMemorySize, lim)) != hipSuccess) return e;
        if ((e = hipFuncSetAttribute((const void *)attention_chunk_kernel<T, D, 16, NW>, hipFuncAttributeMaxDynamicSharedMemorySize, lim)) != hipSuccess) return e;
    }
    if constexpr (NW == 1 || NW == 4) {
        hipError_t e;
        if ((e = hipFuncSetAttribute((const void *)attention_kernel<T, D, 8, NW>, hipFuncAttributeMaxDynamicSharedMemorySize, lim)) != hipSuccess) return e;
        if ((e = hipFuncSetAttribute((const void *)attention_kernel<T, D, 16, NW>, hipFuncAttributeMaxDynamicSharedMemorySize, lim)) != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace

size_t attention_lds_bytes(int S, int d)
{
    const int Sp = round_up(S, 32);
    if (Sp > 256) {                          // one chunk of V^T and of the keys (see attention_chunk_kernel)
        const int ck = round_up(Sp / 2, 32);
        return ((size_t)d * ldv_of(ck) + (size_t)ck * (d + 8)) * sizeof(uint16_t);
    }
    return (size_t)d * ldv_of(Sp) * sizeof(uint16_t);
}

hipError_t attention_init()
{
    hipError_t e;
#define SET(T)                                                         \
    if ((e = set_attr<T, 32, 1>()) != hipSuccess) return e;            \
    if ((e = set_attr<T, 32, 4>()) != hipSuccess) return e;            \
    if ((e = set_attr<T, 64, 1>()) != hipSuccess) return e;            \
    if ((e = set_attr<T, 64, 4>()) != hipSuccess) return e;            \
    if ((e = set_attr<T, 32, 8>()) != hipSuccess) return e;            \
    if ((e = set_attr<T, 64, 8>()) != hipSuccess) return e;
    SET(bf16_t)
    SET(f16_t)
#undef SET
    return hipSuccess;
}

hipError_t launch_attention(const AttnArgs &a, int n_cu, hipStream_t s)
{
    AttnDev d;
    d.qkv = (const uint16_t *)a.qkv; d.y = (uint16_t *)a.y; d.y32 = a.y32;
    d.B = a.B; d.S = a.S; d.Hd = a.Hd; d.heads = a.heads;
    d.Sp = round_up(a.S, 32);
    d.ldv = ldv_of(d.Sp);
    const int D = a.Hd / a.heads;
    d.scale = 1.0f / sqrtf((float)D);
    const size_t lds = attention_lds_bytes(a.S, D);
    // few (batch, head) pairs: one wavefront per workgroup spreads the query blocks over more CUs
    const long wg4 = (long)a.B * a.heads * ((a.S + 63) / 64);
    const bool small = wg4 < n_cu;
    // more than 256 keys (keys staged in LDS chunk by chunk): 128 queries per workgroup when that still gives every
    // other CU a workgroup, else 64
    const bool longseq = d.Sp > 256;
    const bool wide = longseq && 2L * a.B * a.heads * ((a.S + 127) / 128) >= n_cu;
    if (longseq) {
        d.ck = round_up(d.Sp / 2, 32);
        d.nchunks = (d.Sp + d.ck - 1) / d.ck;
        d.ldv = ldv_of(d.ck);
#define GOC(T)                                                                                                   \
        if (D == 32) return wide ? launch_chunked<T, 32, 8>(d, lds, s) : launch_chunked<T, 32, 4>(d, lds, s);      \
        if (D == 64) return wide ? launch_chunked<T, 64, 8>(d, lds, s) : launch_chunked<T, 64, 4>(d, lds, s);
        if (a.dtype == DT_BF16) { GOC(bf16_t) }
        else { GOC(f16_t) }
#undef GOC
        return hipErrorInvalidValue;
    }
#define GO(T)                                                                                  \
    if (D == 32) return small ? launch_d<T, 32, 1>(d, lds, s) : launch_d<T, 32, 4>(d, lds, s); \
    if (D == 64) return small ? launch_d<T, 64, 1>(d, lds, s) : launch_d<T, 64, 4>(d, lds, s);
    if (a.dtype == DT_BF16) { GO(bf16_t) }
    else { GO(f16_t) }
#undef GO
    return hipErrorInvalidValue;
}

}  // namespace eclip
