// Fused dequantize-and-attend decode kernel, matrix-core version (gfx950 MFMA 16x16x32 f16).
//
// Same computation as the vector-ALU kernel (Section 3.1, Eq. 1 over the dequantized cache
// of Section 3.2), reorganised so that the per-element work is done by the matrix cores:
//
//   scores   sum_d q_d (c_td s_d + z_d) = sum_d (q_d s_d) c_td + sum_d q_d z_d
//   output   sum_t p_t (c_td s_tg + z_tg) = sum_t (p_t s_tg) c_td + sum_t p_t z_tg
//
// The integer codes are the B operand.  Masked into the low mantissa bits of an fp16 lane
// they are subnormal halves worth c * 2^-24 (times a power of two that depends on the bit
// position and is folded into the A operand), so "conversion" is one AND per two codes and
// is exact.  The A operand carries q_d s_d (scores) or p_t s_tg (output); to keep fp32-class
// accuracy it is split into a high and a low fp16 part held in rows j and 8 + j of the 16-row
// tile (j = query head within the group, at most 8), and the two partial results are added
// after the MFMA.  The zero-point terms: q . z is one more MFMA per 32 channels (q and z are
// exact in fp16), sum_t p_t z_tg is a handful of fp32 FMAs per block.
//
// A work-group owns one (batch, kv head, split); each of its 4 waves streams every 4th
// 32-token block with the next block's loads in flight, and keeps an online-softmax state.
#include "kvq_internal.h"

namespace kvq {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ half8 as_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    u32x4 v = {a, b, c, d};
    return __builtin_bit_cast(half8, v);
}

__device__ __forceinline__ float half_lo(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu)); }
__device__ __forceinline__ float half_hi(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16)); }

// B operand of MFMA m (8 codes of this lane) straight from the packed dwords: element e of the
// operand is worth code * 2^-24 / code_weight<BITS>(e).
template <int BITS>
__device__ __forceinline__ half8 codes_operand(const uint32_t *dw, int m)
{
    if constexpr (BITS == 8) {
        const uint32_t w0 = dw[2 * m], w1 = dw[2 * m + 1];
        return as_half8(__builtin_amdgcn_perm(0u, w0, 0x0C010C00u), __builtin_amdgcn_perm(0u, w0, 0x0C030C02u),
                        __builtin_amdgcn_perm(0u, w1, 0x0C010C00u), __builtin_amdgcn_perm(0u, w1, 0x0C030C02u));
    } else if constexpr (BITS == 4) {
        const uint32_t x = dw[m], y = x >> 8;
        return as_half8(x & 0x000F000Fu, x & 0x00F000F0u, y & 0x000F000Fu, y & 0x00F000F0u);
    } else {
        const uint32_t x = dw[m >> 1] >> (8 * (m & 1));
        return as_half8(x & 0x00030003u, x & 0x000C000Cu, x & 0x00300030u, x & 0x00C000C0u);
    }
}

// power of two by which the A operand must be divided for element e (the code sits at a
// higher bit position inside its halfword)
template <int BITS>
__device__ __forceinline__ float code_weight_inv(int e)
{
    if (BITS == 8) return 1.0f;
    if (BITS == 4) return ((e >> 1) & 1) ? 0.0625f : 1.0f;
    const int v = (e >> 1) & 3;
    return v == 0 ? 1.0f : v == 1 ? 0.25f : v == 2 ? 0.0625f : 0.015625f;
}

// split two fp32 values into fp16 high parts and (scaled by 2^11) fp16 low parts
__device__ __forceinline__ void split_pair(float r0, float r1, uint32_t &hi, uint32_t &lo)
{
    const half2v h = __builtin_bit_cast(half2v, __builtin_amdgcn_cvt_pkrtz(r0, r1));
    const float d0 = (r0 - (float)h[0]) * 2048.0f, d1 = (r1 - (float)h[1]) * 2048.0f;
    hi = __builtin_bit_cast(uint32_t, h);
    lo = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(d0, d1));
}

template <int KB, int VB>
struct BlockRegs {
    uint32_t kdw[KB < 16 ? 2 * KB : 1];
    uint32_t vdw[VB < 16 ? 2 * VB : 1];
    float2 ks, kz, vs, vz;
};

template <int KB, int VB>
__device__ __forceinline__ void load_block(const DecodeArgs &a, size_t blk_index, int lane, BlockRegs<KB, VB> &r)
{
    if constexpr (KB < 16) {
        const uint8_t *blk = a.lv.kcode + blk_index * block_code_bytes(KB);
#pragma unroll
        for (int c = 0; c < KB / 2; c++) {
            const uint4 x = *reinterpret_cast<const uint4 *>(blk + c * 1024 + lane * 16);
            r.kdw[4 * c] = x.x; r.kdw[4 * c + 1] = x.y; r.kdw[4 * c + 2] = x.z; r.kdw[4 * c + 3] = x.w;
        }
        const float *meta = a.lv.kmeta + blk_index * 256;
        r.ks = *reinterpret_cast<const float2 *>(meta + 2 * lane);
        r.kz = *reinterpret_cast<const float2 *>(meta + kD + 2 * lane);
    }
    if constexpr (VB < 16) {
        const uint8_t *blk = a.lv.vcode + blk_index * block_code_bytes(VB);
#pragma unroll
        for (int c = 0; c < VB / 2; c++) {
            const uint4 x = *reinterpret_cast<const uint4 *>(blk + c * 1024 + lane * 16);
            r.vdw[4 * c] = x.x; r.vdw[4 * c + 1] = x.y; r.vdw[4 * c + 2] = x.z; r.vdw[4 * c + 3] = x.w;
        }
        const float *meta = a.lv.vmeta + blk_index * 256;
        r.vs = *reinterpret_cast<const float2 *>(meta + 2 * lane);          // group lane>>4, tokens 2*(lane&15), +1
        r.vz = *reinterpret_cast<const float2 *>(meta + kD + 2 * lane);
    }
}

template <int KB, int VB, int GQ>
__global__ __launch_bounds__(256) void decode_mfma(DecodeArgs a)
{
    static_assert(GQ == 4 || GQ == 8, "rows j and 8 + j of a 16-row tile");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, rq = lane >> 4;
    const int split = blockIdx.x, bh = blockIdx.y;
    const int b = bh / a.Hkv, h = bh % a.Hkv;
    const int gq_total = a.Hq / a.Hkv;
    const int head0 = blockIdx.z * GQ;
    const int nvalid = gq_total - head0 < GQ ? gq_total - head0 : GQ;
    const size_t qrow0 = (size_t)b * a.Hq + (size_t)h * gq_total + head0;

    __shared__ __attribute__((aligned(16))) _Float16 Ak[4][16][kD + 8];   // score A tiles [row][channel]
    __shared__ __attribute__((aligned(16))) _Float16 Zk[4][kD];           // key zero-points as fp16
    __shared__ __attribute__((aligned(16))) float P[4][GQ][32];           // softmax numerators of the block
    __shared__ __attribute__((aligned(16))) _Float16 Av[4][4][16][32 + 8];// output A tiles [group][row][token]
    __shared__ __attribute__((aligned(16))) float o_lds[4][GQ][kD];
    __shared__ float az_lds[4][GQ][4];
    __shared__ float ml_lds[4][GQ][2];

    // rows that are never written must read as zero
    for (int i = tid; i < 4 * 16 * (kD + 8) / 2; i += 256) reinterpret_cast<uint32_t *>(&Ak[0][0][0])[i] = 0u;
    for (int i = tid; i < 4 * 4 * 16 * (32 + 8) / 2; i += 256) reinterpret_cast<uint32_t *>(&Av[0][0][0][0])[i] = 0u;

    // ---- query setup: exact fp16 tiles for the q.z and fp16-row MFMAs, scaled fp32 pairs for q*s
    const float c = a.scale_log2e;
    float qraw[GQ][2];
    float qmax = 0.0f;
#pragma unroll
    for (int j = 0; j < GQ; j++) {
        uint32_t w = 0;
        if (j < nvalid) w = *reinterpret_cast<const uint32_t *>(a.q + (qrow0 + j) * kD + 2 * lane);
        qraw[j][0] = half_lo(w) * c;
        qraw[j][1] = half_hi(w) * c;
        qmax = fmaxf(qmax, fmaxf(fabsf(qraw[j][0]), fabsf(qraw[j][1])));
    }
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) qmax = fmaxf(qmax, __shfl_xor(qmax, s));
    int qexp = 0;
    if (qmax > 0.0f) (void)frexpf(qmax, &qexp);          // qmax = f * 2^qexp, f in [0.5, 1)
    const float alpha_h = ldexpf(1.0f, 24 + qexp);        // undo 2^-24 of the codes and 2^-qexp of q
    const float alpha_l = ldexpf(1.0f, 13 + qexp);
    float q2[GQ][2];
#pragma unroll
    for (int j = 0; j < GQ; j++) {
        q2[j][0] = ldexpf(qraw[j][0], -qexp) * code_weight_inv<KB < 16 ? KB : 8>((2 * lane) & 7);
        q2[j][1] = ldexpf(qraw[j][1], -qexp) * code_weight_inv<KB < 16 ? KB : 8>((2 * lane + 1) & 7);
    }
    half8 Aq[4];
    {
        const int jr = n & 7;
#pragma unroll
        for (int cb = 0; cb < 4; cb++) {
            uint4 x = make_uint4(0, 0, 0, 0);
            if (jr < nvalid) x = *reinterpret_cast<const uint4 *>(a.q + (qrow0 + jr) * kD + 32 * cb + 8 * rq);
            Aq[cb] = as_half8(x.x, x.y, x.z, x.w);
        }
    }
    const float vw0 = code_weight_inv<VB < 16 ? VB : 8>((2 * n) & 7), vw1 = code_weight_inv<VB < 16 ? VB : 8>((2 * n + 1) & 7);
    __syncthreads();

    float m[4], l[4];
    float4v O[8];
    float oF[GQ][2], accz[GQ];
#pragma unroll
    for (int i = 0; i < 4; i++) { m[i] = -INFINITY; l[i] = 0.0f; }
#pragma unroll
    for (int cblk = 0; cblk < 8; cblk++) O[cblk] = float4v{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int j = 0; j < GQ; j++) { oF[j][0] = oF[j][1] = 0.0f; accz[j] = 0.0f; }

    const int units = a.n_blocks + (a.n_res + 31) / 32;
    const int u0 = split * a.units_per_split;
    const int u1 = u0 + a.units_per_split < units ? u0 + a.units_per_split : units;

    BlockRegs<KB, VB> cur, nxt;
    if (u0 + wave < u1 && u0 + wave < a.n_blocks) load_block<KB, VB>(a, (size_t)bh * a.NB + u0 + wave, lane, cur);

    for (int u = u0 + wave; u < u1; u += 4) {
        const bool packed = u < a.n_blocks;
        const int pos0 = packed ? u * kG : a.n_blocks * kG + (u - a.n_blocks) * 32;
        const int nt = packed ? 32 : (a.n_res - (u - a.n_blocks) * 32 < 32 ? a.n_res - (u - a.n_blocks) * 32 : 32);
        if (u + 4 < u1 && u + 4 < a.n_blocks) load_block<KB, VB>(a, (size_t)bh * a.NB + u + 4, lane, nxt);

        // ------------------------------------------------ scores
        float s[2][4];
        bool k_rows = true;
        if constexpr (KB < 16) if (packed) {
            k_rows = false;
#pragma unroll
            for (int j = 0; j < GQ; j++) {
                uint32_t hi, lo;
                split_pair(q2[j][0] * cur.ks.x, q2[j][1] * cur.ks.y, hi, lo);
                *reinterpret_cast<uint32_t *>(&Ak[wave][j][2 * lane]) = hi;
                *reinterpret_cast<uint32_t *>(&Ak[wave][8 + j][2 * lane]) = lo;
            }
            *reinterpret_cast<uint32_t *>(&Zk[wave][2 * lane]) = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(cur.kz.x, cur.kz.y));
            wave_lds_sync();
            float4v S0 = {0.0f, 0.0f, 0.0f, 0.0f}, S1 = S0, Z = S0;
#pragma unroll
            for (int cb = 0; cb < 4; cb++) {
                const half8 Aop = *reinterpret_cast<const half8 *>(&Ak[wave][n][32 * cb + 8 * rq]);
                const half8 Bz = *reinterpret_cast<const half8 *>(&Zk[wave][32 * cb + 8 * rq]);
                S0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(Aop, codes_operand<KB>(cur.kdw, cb), S0, 0, 0, 0);
                S1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(Aop, codes_operand<KB>(cur.kdw, 4 + cb), S1, 0, 0, 0);
                Z = __builtin_amdgcn_mfma_f32_16x16x32_f16(Aq[cb], Bz, Z, 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const float o0 = __shfl_xor(S0[i], 32), o1 = __shfl_xor(S1[i], 32);
                const float h0 = rq < 2 ? S0[i] : o0, l0 = rq < 2 ? o0 : S0[i];
                const float h1 = rq < 2 ? S1[i] : o1, l1 = rq < 2 ? o1 : S1[i];
                s[0][i] = fmaf(alpha_h, h0, fmaf(alpha_l, l0, c * Z[i]));
                s[1][i] = fmaf(alpha_h, h1, fmaf(alpha_l, l1, c * Z[i]));
            }
        }
        if (k_rows) {
            float4v S0 = {0.0f, 0.0f, 0.0f, 0.0f}, S1 = S0;
            const uint16_t *row0, *row1;
            {
                const int p0 = pos0 + n, p1 = pos0 + 16 + n;
                row0 = packed ? reinterpret_cast<const uint16_t *>(a.lv.kcode) + ((size_t)bh * a.NB * kG + p0) * kD
                              : a.lv.kres + ((size_t)bh * a.RC + p0 % a.RC) * kD;
                row1 = packed ? reinterpret_cast<const uint16_t *>(a.lv.kcode) + ((size_t)bh * a.NB * kG + p1) * kD
                              : a.lv.kres + ((size_t)bh * a.RC + p1 % a.RC) * kD;
            }
#pragma unroll
            for (int cb = 0; cb < 4; cb++) {
                uint4 x0 = make_uint4(0, 0, 0, 0), x1 = x0;
                if (n < nt) x0 = *reinterpret_cast<const uint4 *>(row0 + 32 * cb + 8 * rq);
                if (16 + n < nt) x1 = *reinterpret_cast<const uint4 *>(row1 + 32 * cb + 8 * rq);
                S0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(Aq[cb], as_half8(x0.x, x0.y, x0.z, x0.w), S0, 0, 0, 0);
                S1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(Aq[cb], as_half8(x1.x, x1.y, x1.z, x1.w), S1, 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < 4; i++) {
                s[0][i] = n < nt ? c * S0[i] : -INFINITY;
                s[1][i] = 16 + n < nt ? c * S1[i] : -INFINITY;
            }
        }

        // ------------------------------------------------ online softmax (log2 domain), rows 4*rq + i
        float mnew[4];
        bool grew = false;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            float mb = fmaxf(s[0][i], s[1][i]);
            mb = fmaxf(mb, __shfl_xor(mb, 1));
            mb = fmaxf(mb, __shfl_xor(mb, 2));
            mb = fmaxf(mb, __shfl_xor(mb, 4));
            mb = fmaxf(mb, __shfl_xor(mb, 8));
            mnew[i] = fmaxf(m[i], mb);
            grew = grew || (mnew[i] > m[i]);
        }
        if (__any(grew)) {
            float alpha[4];
#pragma unroll
            for (int i = 0; i < 4; i++) {
                alpha[i] = exp2f(m[i] - mnew[i]);
                l[i] *= alpha[i];
                m[i] = mnew[i];
            }
#pragma unroll
            for (int cblk = 0; cblk < 8; cblk++)
#pragma unroll
                for (int i = 0; i < 4; i++) O[cblk][i] *= alpha[i];
#pragma unroll
            for (int j = 0; j < GQ; j++) {
                const float aj = __shfl(alpha[j & 3], 16 * (j >> 2));
                oF[j][0] *= aj; oF[j][1] *= aj; accz[j] *= aj;
            }
        }
        float p[2][4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            p[0][i] = exp2f(s[0][i] - m[i]);
            p[1][i] = exp2f(s[1][i] - m[i]);
            l[i] += p[0][i] + p[1][i];
        }
        if (rq < 2) {
#pragma unroll
            for (int i = 0; i < 4; i++) {
                if (4 * rq + i < GQ) {
                    P[wave][(4 * rq + i) % GQ][n] = p[0][i];
                    P[wave][(4 * rq + i) % GQ][16 + n] = p[1][i];
                }
            }
        }
        wave_lds_sync();

        // ------------------------------------------------ output
        bool v_rows = true;
        if constexpr (VB < 16) if (packed) {
            v_rows = false;
            const float sv0 = cur.vs.x * vw0, sv1 = cur.vs.y * vw1;
#pragma unroll
            for (int j = 0; j < GQ; j++) {
                const float2 pp = *reinterpret_cast<const float2 *>(&P[wave][j][2 * n]);
                uint32_t hi, lo;
                split_pair(pp.x * sv0, pp.y * sv1, hi, lo);
                *reinterpret_cast<uint32_t *>(&Av[wave][rq][j][2 * n]) = hi;
                *reinterpret_cast<uint32_t *>(&Av[wave][rq][8 + j][2 * n]) = lo;
                accz[j] = fmaf(pp.x, cur.vz.x, fmaf(pp.y, cur.vz.y, accz[j]));
            }
            wave_lds_sync();
            half8 Aop[4];
#pragma unroll
            for (int gd = 0; gd < 4; gd++) Aop[gd] = *reinterpret_cast<const half8 *>(&Av[wave][gd][n][8 * rq]);
#pragma unroll
            for (int cblk = 0; cblk < 8; cblk++)
                O[cblk] = __builtin_amdgcn_mfma_f32_16x16x32_f16(Aop[cblk >> 1], codes_operand<VB>(cur.vdw, cblk), O[cblk], 0, 0, 0);
        }
        if (v_rows) {
            // fp16 rows (the 16-bit region or the window ring): lane owns channels 2*lane, 2*lane+1
            for (int tt = 0; tt < nt; tt++) {
                const int pos = pos0 + tt;
                const uint16_t *row = packed ? reinterpret_cast<const uint16_t *>(a.lv.vcode) + ((size_t)bh * a.NB * kG + pos) * kD
                                             : a.lv.vres + ((size_t)bh * a.RC + pos % a.RC) * kD;
                const uint32_t x = *reinterpret_cast<const uint32_t *>(row + 2 * lane);
                const float v0 = half_lo(x), v1 = half_hi(x);
#pragma unroll
                for (int j = 0; j < GQ; j++) {
                    const float pj = P[wave][j][tt];
                    oF[j][0] = fmaf(pj, v0, oF[j][0]);
                    oF[j][1] = fmaf(pj, v1, oF[j][1]);
                }
            }
        }
        wave_lds_sync();
        cur = nxt;
    }

    // ---------------------------------------------------- wave results -> LDS
#pragma unroll
    for (int i = 0; i < 4; i++) {
        l[i] += __shfl_xor(l[i], 1); l[i] += __shfl_xor(l[i], 2);
        l[i] += __shfl_xor(l[i], 4); l[i] += __shfl_xor(l[i], 8);
    }
#pragma unroll
    for (int j = 0; j < GQ; j++) {
        accz[j] += __shfl_xor(accz[j], 1); accz[j] += __shfl_xor(accz[j], 2);
        accz[j] += __shfl_xor(accz[j], 4); accz[j] += __shfl_xor(accz[j], 8);
        if (n == 0) az_lds[wave][j][rq] = accz[j];
    }
    const float two24 = 16777216.0f, two13 = 8192.0f;
    if (rq < 2) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
            if (4 * rq + i < GQ) {
                const int j = (4 * rq + i) % GQ;
#pragma unroll
                for (int cblk = 0; cblk < 8; cblk++) o_lds[wave][j][16 * cblk + n] = two24 * O[cblk][i];
                if (n == 0) { ml_lds[wave][j][0] = m[i]; ml_lds[wave][j][1] = l[i]; }
            }
        }
    }
    wave_lds_sync();
    if (rq >= 2) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
            if (4 * (rq - 2) + i < GQ) {
                const int j = (4 * (rq - 2) + i) % GQ;
#pragma unroll
                for (int cblk = 0; cblk < 8; cblk++) o_lds[wave][j][16 * cblk + n] += two13 * O[cblk][i];
            }
        }
    }
    wave_lds_sync();
#pragma unroll
    for (int j = 0; j < GQ; j++) {
        o_lds[wave][j][2 * lane] += oF[j][0];
        o_lds[wave][j][2 * lane + 1] += oF[j][1];
    }
    __syncthreads();

    // ---------------------------------------------------- merge the 4 waves, write the split's partial
    for (int i = tid; i < nvalid * kD; i += 256) {
        const int j = i / kD, d = i % kD;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; w++) M = fmaxf(M, ml_lds[w][j][0]);
        float L = 0.0f, Osum = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; w++) {
            const float mw = ml_lds[w][j][0];
            const float f = mw == -INFINITY ? 0.0f : exp2f(mw - M);
            L = fmaf(ml_lds[w][j][1], f, L);
            Osum = fmaf(o_lds[w][j][d] + az_lds[w][j][d >> 5], f, Osum);
        }
        const size_t prow = (qrow0 + j) * a.splits + split;
        a.part_o[prow * kD + d] = Osum;
        if (d == 0) { a.part_ml[prow * 2] = M; a.part_ml[prow * 2 + 1] = L; }
    }
}

template <int KB, int VB>
hipError_t launch_gq(const DecodeArgs &a, hipStream_t s)
{
    const int gq = a.Hq / a.Hkv;
    const int BH = a.B * a.Hkv;
    const dim3 block(256);
    if (gq <= 4) {
        hipLaunchKernelGGL((decode_mfma<KB, VB, 4>), dim3(a.splits, BH, 1), block, 0, s, a);
    } else {
        hipLaunchKernelGGL((decode_mfma<KB, VB, 8>), dim3(a.splits, BH, (gq + 7) / 8), block, 0, s, a);
    }
    return hipGetLastError();
}

template <int KB>
hipError_t launch_vb(const DecodeArgs &a, hipStream_t s)
{
    switch (a.lv.vbits) {
    case 2: return launch_gq<KB, 2>(a, s);
    case 4: return launch_gq<KB, 4>(a, s);
    case 8: return launch_gq<KB, 8>(a, s);
    default: return launch_gq<KB, 16>(a, s);
    }
}

}  // namespace

hipError_t launch_decode_mfma(const DecodeArgs &a, hipStream_t s)
{
    if (a.B * a.Hkv > 65535) return hipErrorInvalidConfiguration;
    switch (a.lv.kbits) {
    case 2: return launch_vb<2>(a, s);
    case 4: return launch_vb<4>(a, s);
    case 8: return launch_vb<8>(a, s);
    default: return launch_vb<16>(a, s);
    }
}

}  // namespace kvq
