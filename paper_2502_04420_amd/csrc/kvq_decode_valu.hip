// Fused dequantize-and-attend decode kernel, vector-ALU version, and the split combine.
//
// Section 3.1, Eq. 1 of the paper over the dequantized cache of Section 3.2
// (X^ = Q(X) s + z): for one (batch, kv head) a work-group streams a range of 32-token
// blocks; each of its 4 waves owns every 4th block and keeps an online-softmax state
// (running max, sum, un-normalised output) for the GQ query heads that share the kv
// head.  Codes are unpacked in registers, dequantized with one fma and consumed at
// once; nothing dequantized is written back.  Partial states of the waves are merged
// in LDS, those of the splits by combine_splits.
#include "kvq_internal.h"

namespace kvq {
namespace {

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ float half_lo(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu)); }
__device__ __forceinline__ float half_hi(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16)); }

// a block's metadata (128 scales, fp32 or fp16; 128 fp16 zero-points) into an LDS tile of 256 floats, one wave
__device__ __forceinline__ void stage_meta(const float *meta, bool narrow, float *tile, int lane)
{
    if (lane < 32) {
        if (narrow) {
            const uint2 h = *reinterpret_cast<const uint2 *>(meta_scales16(meta) + 4 * lane);
            *reinterpret_cast<float4 *>(&tile[4 * lane]) = make_float4(half_lo(h.x), half_hi(h.x), half_lo(h.y), half_hi(h.y));
        } else {
            *reinterpret_cast<float4 *>(&tile[4 * lane]) = *reinterpret_cast<const float4 *>(meta + 4 * lane);
        }
    } else {
        const uint2 z = *reinterpret_cast<const uint2 *>(meta_zeros(meta, narrow) + 4 * (lane - 32));
        *reinterpret_cast<float4 *>(&tile[kD + 4 * (lane - 32)]) = make_float4(half_lo(z.x), half_hi(z.x), half_lo(z.y), half_hi(z.y));
    }
}

template <int BITS>
__device__ __forceinline__ float code_as_float(const uint32_t *dw, int ci)
{
    return (float)((dw[code_dword<BITS>(ci)] >> code_shift<BITS>(ci)) & ((1u << BITS) - 1u));
}

template <int KB, int VB, int GQ, bool KPT>
__global__ __launch_bounds__(256) void decode_valu(DecodeArgs a)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, kq = lane >> 4;
    const int split = blockIdx.x, bh = blockIdx.y;
    const int b = bh / a.Hkv, h = bh % a.Hkv;
    const int gq_total = a.Hq / a.Hkv;
    const int head0 = blockIdx.z * GQ;
    const int nvalid = gq_total - head0 < GQ ? gq_total - head0 : GQ;
    const size_t qrow0 = (size_t)b * a.Hq + (size_t)h * gq_total + head0;

    __shared__ __attribute__((aligned(16))) float q_lds[GQ][kD];
    __shared__ __attribute__((aligned(16))) float kmeta_lds[4][256];
    __shared__ __attribute__((aligned(16))) float vmeta_lds[4][256];
    __shared__ __attribute__((aligned(16))) float p_lds[4][GQ][32];
    __shared__ __attribute__((aligned(16))) float o_lds[4][GQ][kD];
    __shared__ float ml_lds[4][GQ][2];

    for (int i = tid; i < GQ * kD; i += 256) {
        const int j = i / kD, d = i % kD;
        q_lds[j][d] = j < nvalid ? (float)__builtin_bit_cast(_Float16, a.q[(qrow0 + j) * kD + d]) * a.scale_log2e : 0.0f;
    }
    __syncthreads();

    float m[GQ], l[GQ], oP[GQ][8], oF[GQ][2];
#pragma unroll
    for (int j = 0; j < GQ; j++) {
        m[j] = -INFINITY; l[j] = 0.0f; oF[j][0] = oF[j][1] = 0.0f;
#pragma unroll
        for (int c = 0; c < 8; c++) oP[j][c] = 0.0f;
    }

    int u0, u1;
    split_range(a, split, u0, u1);

    for (int u = u0 + wave; u < u1; u += 4) {
        const bool packed = u < a.n_blocks;
        const int pos0 = packed ? u * kG : a.n_blocks * kG + (u - a.n_blocks) * 32;
        const int nt = packed ? 32 : (a.n_res - (u - a.n_blocks) * 32 < 32 ? a.n_res - (u - a.n_blocks) * 32 : 32);
        const size_t blk_index = (size_t)bh * a.NB + u;

        // ------------------------------------------------ scores: q . k^ for the block's tokens
        float acc[GQ][2];
#pragma unroll
        for (int j = 0; j < GQ; j++) acc[j][0] = acc[j][1] = 0.0f;

        bool k_rows = true;
        if constexpr (KB < 16) if (packed) {
            k_rows = false;
            constexpr int NDW = 2 * KB;
            uint32_t dw[NDW];
            const uint8_t *blk = a.lv.kcode + blk_index * block_code_bytes(KB);
#pragma unroll
            for (int c = 0; c < NDW / 4; c++) {
                const uint4 x = *reinterpret_cast<const uint4 *>(blk + c * 1024 + lane * 16);
                dw[4 * c] = x.x; dw[4 * c + 1] = x.y; dw[4 * c + 2] = x.z; dw[4 * c + 3] = x.w;
            }
            stage_meta(a.lv.kmeta + blk_index * meta_words(a.lv.narrow != 0), a.lv.narrow != 0, kmeta_lds[wave], lane);
            wave_lds_sync();
#pragma unroll
            for (int cb = 0; cb < 4; cb++) {
                const int ch0 = 32 * cb + 8 * kq;
                float s8[8], z8[8], k0[8], k1[8];
                *reinterpret_cast<float4 *>(&s8[0]) = *reinterpret_cast<const float4 *>(&kmeta_lds[wave][ch0]);
                *reinterpret_cast<float4 *>(&s8[4]) = *reinterpret_cast<const float4 *>(&kmeta_lds[wave][ch0 + 4]);
                *reinterpret_cast<float4 *>(&z8[0]) = *reinterpret_cast<const float4 *>(&kmeta_lds[wave][kD + ch0]);
                *reinterpret_cast<float4 *>(&z8[4]) = *reinterpret_cast<const float4 *>(&kmeta_lds[wave][kD + ch0 + 4]);
                if constexpr (KPT) {
                    // keys grouped per token: one (s, z) per token and 32-channel group cb, stored at [group][token]
                    const float s0 = kmeta_lds[wave][32 * cb + n], s1 = kmeta_lds[wave][32 * cb + 16 + n];
                    const float z0 = kmeta_lds[wave][kD + 32 * cb + n], z1 = kmeta_lds[wave][kD + 32 * cb + 16 + n];
#pragma unroll
                    for (int e = 0; e < 8; e++) {
                        k0[e] = fmaf(code_as_float<KB>(dw, 8 * cb + e), s0, z0);
                        k1[e] = fmaf(code_as_float<KB>(dw, 8 * (4 + cb) + e), s1, z1);
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 8; e++) {
                        k0[e] = fmaf(code_as_float<KB>(dw, 8 * cb + e), s8[e], z8[e]);
                        k1[e] = fmaf(code_as_float<KB>(dw, 8 * (4 + cb) + e), s8[e], z8[e]);
                    }
                }
#pragma unroll
                for (int j = 0; j < GQ; j++) {
                    float q8[8];
                    *reinterpret_cast<float4 *>(&q8[0]) = *reinterpret_cast<const float4 *>(&q_lds[j][ch0]);
                    *reinterpret_cast<float4 *>(&q8[4]) = *reinterpret_cast<const float4 *>(&q_lds[j][ch0 + 4]);
#pragma unroll
                    for (int e = 0; e < 8; e++) {
                        acc[j][0] = fmaf(q8[e], k0[e], acc[j][0]);
                        acc[j][1] = fmaf(q8[e], k1[e], acc[j][1]);
                    }
                }
            }
        }
        if (k_rows) {
            // fp16 rows: the 16-bit region or the window ring
            const uint16_t *row[2];
#pragma unroll
            for (int th = 0; th < 2; th++) {
                const int pos = pos0 + 16 * th + n;
                row[th] = packed ? reinterpret_cast<const uint16_t *>(a.lv.kcode) + ((size_t)bh * a.NB * kG + pos) * kD
                                 : a.lv.kres + ((size_t)bh * a.RC + pos % a.RC) * kD;
            }
#pragma unroll
            for (int cb = 0; cb < 4; cb++) {
                const int ch0 = 32 * cb + 8 * kq;
                float kf[2][8];
#pragma unroll
                for (int th = 0; th < 2; th++) {
                    uint4 x = make_uint4(0, 0, 0, 0);
                    if (16 * th + n < nt) x = *reinterpret_cast<const uint4 *>(row[th] + ch0);
                    kf[th][0] = half_lo(x.x); kf[th][1] = half_hi(x.x); kf[th][2] = half_lo(x.y); kf[th][3] = half_hi(x.y);
                    kf[th][4] = half_lo(x.z); kf[th][5] = half_hi(x.z); kf[th][6] = half_lo(x.w); kf[th][7] = half_hi(x.w);
                }
#pragma unroll
                for (int j = 0; j < GQ; j++) {
                    float q8[8];
                    *reinterpret_cast<float4 *>(&q8[0]) = *reinterpret_cast<const float4 *>(&q_lds[j][ch0]);
                    *reinterpret_cast<float4 *>(&q8[4]) = *reinterpret_cast<const float4 *>(&q_lds[j][ch0 + 4]);
#pragma unroll
                    for (int e = 0; e < 8; e++) {
                        acc[j][0] = fmaf(q8[e], kf[0][e], acc[j][0]);
                        acc[j][1] = fmaf(q8[e], kf[1][e], acc[j][1]);
                    }
                }
            }
        }

        // ------------------------------------------------ online softmax (log2 domain)
#pragma unroll
        for (int j = 0; j < GQ; j++) {
            float s0 = acc[j][0], s1 = acc[j][1];
            s0 += __shfl_xor(s0, 16); s1 += __shfl_xor(s1, 16);
            s0 += __shfl_xor(s0, 32); s1 += __shfl_xor(s1, 32);
            if (n >= nt) s0 = -INFINITY;
            if (16 + n >= nt) s1 = -INFINITY;
            float mx = fmaxf(s0, s1);
            mx = fmaxf(mx, __shfl_xor(mx, 1));
            mx = fmaxf(mx, __shfl_xor(mx, 2));
            mx = fmaxf(mx, __shfl_xor(mx, 4));
            mx = fmaxf(mx, __shfl_xor(mx, 8));
            const float m_new = fmaxf(m[j], mx);
            const float alpha = exp2f(m[j] - m_new);
            const float p0 = exp2f(s0 - m_new), p1 = exp2f(s1 - m_new);
            l[j] = l[j] * alpha + (p0 + p1);
            m[j] = m_new;
            oF[j][0] *= alpha; oF[j][1] *= alpha;
#pragma unroll
            for (int c = 0; c < 8; c++) oP[j][c] *= alpha;
            if (kq == 0) { p_lds[wave][j][n] = p0; p_lds[wave][j][16 + n] = p1; }
        }
        wave_lds_sync();

        // ------------------------------------------------ output: sum_t p_t v^_t
        bool v_rows = true;
        if constexpr (VB < 16) if (packed) {
            v_rows = false;
            constexpr int NDW = 2 * VB;
            uint32_t dw[NDW];
            const uint8_t *blk = a.lv.vcode + blk_index * block_code_bytes(VB);
#pragma unroll
            for (int c = 0; c < NDW / 4; c++) {
                const uint4 x = *reinterpret_cast<const uint4 *>(blk + c * 1024 + lane * 16);
                dw[4 * c] = x.x; dw[4 * c + 1] = x.y; dw[4 * c + 2] = x.z; dw[4 * c + 3] = x.w;
            }
            stage_meta(a.lv.vmeta + blk_index * meta_words(a.lv.narrow != 0), a.lv.narrow != 0, vmeta_lds[wave], lane);
            wave_lds_sync();
            float sv[4][8], zv[4][8];     // [channel group][token 8*kq + e]
#pragma unroll
            for (int gd = 0; gd < 4; gd++) {
                *reinterpret_cast<float4 *>(&sv[gd][0]) = *reinterpret_cast<const float4 *>(&vmeta_lds[wave][32 * gd + 8 * kq]);
                *reinterpret_cast<float4 *>(&sv[gd][4]) = *reinterpret_cast<const float4 *>(&vmeta_lds[wave][32 * gd + 8 * kq + 4]);
                *reinterpret_cast<float4 *>(&zv[gd][0]) = *reinterpret_cast<const float4 *>(&vmeta_lds[wave][kD + 32 * gd + 8 * kq]);
                *reinterpret_cast<float4 *>(&zv[gd][4]) = *reinterpret_cast<const float4 *>(&vmeta_lds[wave][kD + 32 * gd + 8 * kq + 4]);
            }
            float p8[GQ][8];
#pragma unroll
            for (int j = 0; j < GQ; j++) {
                *reinterpret_cast<float4 *>(&p8[j][0]) = *reinterpret_cast<const float4 *>(&p_lds[wave][j][8 * kq]);
                *reinterpret_cast<float4 *>(&p8[j][4]) = *reinterpret_cast<const float4 *>(&p_lds[wave][j][8 * kq + 4]);
            }
#pragma unroll
            for (int cblk = 0; cblk < 8; cblk++) {
                float vh[8];
#pragma unroll
                for (int e = 0; e < 8; e++)
                    vh[e] = fmaf(code_as_float<VB>(dw, 8 * cblk + e), sv[cblk >> 1][e], zv[cblk >> 1][e]);
#pragma unroll
                for (int j = 0; j < GQ; j++)
#pragma unroll
                    for (int e = 0; e < 8; e++) oP[j][cblk] = fmaf(p8[j][e], vh[e], oP[j][cblk]);
            }
        }
        if (v_rows) {
            // fp16 rows: lane owns channels 2*lane, 2*lane+1
            for (int tt = 0; tt < nt; tt++) {
                const int pos = pos0 + tt;
                const uint16_t *row = packed ? reinterpret_cast<const uint16_t *>(a.lv.vcode) + ((size_t)bh * a.NB * kG + pos) * kD
                                             : a.lv.vres + ((size_t)bh * a.RC + pos % a.RC) * kD;
                const uint32_t x = *reinterpret_cast<const uint32_t *>(row + 2 * lane);
                const float v0 = half_lo(x), v1 = half_hi(x);
#pragma unroll
                for (int j = 0; j < GQ; j++) {
                    const float p = p_lds[wave][j][tt];
                    oF[j][0] = fmaf(p, v0, oF[j][0]);
                    oF[j][1] = fmaf(p, v1, oF[j][1]);
                }
            }
        }
        wave_lds_sync();   // p_lds / meta tiles are rewritten by the next unit
    }

    // ---------------------------------------------------- merge the 4 waves, write the split's partial
#pragma unroll
    for (int j = 0; j < GQ; j++) {
        l[j] += __shfl_xor(l[j], 1); l[j] += __shfl_xor(l[j], 2);
        l[j] += __shfl_xor(l[j], 4); l[j] += __shfl_xor(l[j], 8);
#pragma unroll
        for (int c = 0; c < 8; c++) {
            oP[j][c] += __shfl_xor(oP[j][c], 16);
            oP[j][c] += __shfl_xor(oP[j][c], 32);
        }
        if (kq == 0) {
#pragma unroll
            for (int c = 0; c < 8; c++) o_lds[wave][j][16 * c + n] = oP[j][c];
        }
        if (lane == 0) { ml_lds[wave][j][0] = m[j]; ml_lds[wave][j][1] = l[j]; }
    }
    wave_lds_sync();
#pragma unroll
    for (int j = 0; j < GQ; j++) {
        o_lds[wave][j][2 * lane] += oF[j][0];
        o_lds[wave][j][2 * lane + 1] += oF[j][1];
    }
    __syncthreads();
    for (int i = tid; i < nvalid * kD; i += 256) {
        const int j = i / kD, d = i % kD;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; w++) M = fmaxf(M, ml_lds[w][j][0]);
        float L = 0.0f, O = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; w++) {
            const float mw = ml_lds[w][j][0];
            const float f = mw == -INFINITY ? 0.0f : exp2f(mw - M);
            L = fmaf(ml_lds[w][j][1], f, L);
            O = fmaf(o_lds[w][j][d], f, O);
        }
        const size_t prow = (qrow0 + j) * a.splits + split;
        a.part_o[prow * kD + d] = O;
        if (d == 0) { a.part_ml[prow * 2] = M; a.part_ml[prow * 2 + 1] = L; }
    }
}

// Merge the splits of one (batch, query head) by log-sum-exp and store fp16 (round to nearest even).
// 512 threads: thread = (quarter g, channel d).  Quarter g merges the splits g, g + 4, g + 8, .., fetching
// W partial records at a time with independent loads (a plain loop would pay one memory latency per
// split; W = 16 for more than 32 splits, so that up to 64 splits are one round trip); the four quarter results are
// merged through LDS.  The order of all sums is fixed.
template <int W>
__global__ __launch_bounds__(512) void combine_splits(DecodeArgs a)
{
    const size_t row = blockIdx.x;
    const int d = threadIdx.x & 127, g = threadIdx.x >> 7;
    const float *ml = a.part_ml + row * a.splits * 2;
    const float *po = a.part_o + row * a.splits * kD + d;
    __shared__ float Mq[4], Lq[4], Oq[4][kD];
    float M = -INFINITY, L = 0.0f, O = 0.0f;
    for (int s0 = g; s0 < a.splits; s0 += 4 * W) {
        float m8[W], l8[W], o8[W];
#pragma unroll
        for (int k = 0; k < W; k++) {
            const int sp = s0 + 4 * k;
            const bool ok = sp < a.splits;
            m8[k] = ok ? ml[sp * 2] : -INFINITY;
            l8[k] = ok ? ml[sp * 2 + 1] : 0.0f;
            o8[k] = ok ? po[(size_t)sp * kD] : 0.0f;
        }
        float Mn = M;
#pragma unroll
        for (int k = 0; k < W; k++) Mn = fmaxf(Mn, m8[k]);
        const float fo = exp2f(M - Mn);          // M = -inf on the first pass: factor 0 on empty sums
        L *= fo; O *= fo;
#pragma unroll
        for (int k = 0; k < W; k++) {
            const float f = exp2f(m8[k] - Mn);   // an absent split has m = -inf: factor 0
            L = fmaf(l8[k], f, L);
            O = fmaf(o8[k], f, O);
        }
        M = Mn;
    }
    Oq[g][d] = O;
    if (d == 0) { Mq[g] = M; Lq[g] = L; }
    __syncthreads();
    if (g == 0) {
        const float Mt = fmaxf(fmaxf(Mq[0], Mq[1]), fmaxf(Mq[2], Mq[3]));      // quarter 0 always holds split 0: finite
        float Lt = 0.0f, Ot = 0.0f;
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const float f = exp2f(Mq[k] - Mt);   // an empty quarter has M = -inf: factor 0
            Lt = fmaf(Lq[k], f, Lt);
            Ot = fmaf(Oq[k][d], f, Ot);
        }
        a.out[row * kD + d] = __builtin_bit_cast(uint16_t, (_Float16)(Ot / Lt));
    }
}

template <int KB, int VB, bool KPT>
hipError_t launch_gq(const DecodeArgs &a, hipStream_t s)
{
    const int gq = a.Hq / a.Hkv;
    const int BH = a.B * a.Hkv;
    const dim3 block(256);
    if (gq == 1) {
        hipLaunchKernelGGL((decode_valu<KB, VB, 1, KPT>), dim3(a.splits, BH, 1), block, 0, s, a);
    } else if (gq == 2) {
        hipLaunchKernelGGL((decode_valu<KB, VB, 2, KPT>), dim3(a.splits, BH, 1), block, 0, s, a);
    } else if (gq <= 4) {
        hipLaunchKernelGGL((decode_valu<KB, VB, 4, KPT>), dim3(a.splits, BH, 1), block, 0, s, a);
    } else {
        hipLaunchKernelGGL((decode_valu<KB, VB, 8, KPT>), dim3(a.splits, BH, (gq + 7) / 8), block, 0, s, a);
    }
    return hipGetLastError();
}

template <int KB, bool KPT>
hipError_t launch_vb(const DecodeArgs &a, hipStream_t s)
{
    switch (a.lv.vbits) {
    case 2: return launch_gq<KB, 2, KPT>(a, s);
    case 4: return launch_gq<KB, 4, KPT>(a, s);
    case 8: return launch_gq<KB, 8, KPT>(a, s);
    default: return launch_gq<KB, 16, KPT>(a, s);
    }
}

}  // namespace

hipError_t launch_decode_valu(const DecodeArgs &a, hipStream_t s)
{
    if (a.B * a.Hkv > 65535) return hipErrorInvalidConfiguration;
    if (a.lv.kpt) {                 // the key grouping only matters for quantized keys
        switch (a.lv.kbits) {
        case 2: return launch_vb<2, true>(a, s);
        case 4: return launch_vb<4, true>(a, s);
        case 8: return launch_vb<8, true>(a, s);
        default: break;
        }
    }
    switch (a.lv.kbits) {
    case 2: return launch_vb<2, false>(a, s);
    case 4: return launch_vb<4, false>(a, s);
    case 8: return launch_vb<8, false>(a, s);
    default: return launch_vb<16, false>(a, s);
    }
}

hipError_t launch_combine(const DecodeArgs &a, hipStream_t s)
{
    if (a.splits > 32) hipLaunchKernelGGL(combine_splits<16>, dim3(a.B * a.Hq), dim3(512), 0, s, a);
    else hipLaunchKernelGGL(combine_splits<8>, dim3(a.B * a.Hq), dim3(512), 0, s, a);
    return hipGetLastError();
}

}  // namespace kvq
