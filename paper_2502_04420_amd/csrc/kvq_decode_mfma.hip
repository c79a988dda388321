// Fused dequantize-and-attend decode kernel, matrix-core version (gfx950 MFMA 16x16x32 f16).
//
// Same computation as the vector-ALU kernel (Section 3.1, Eq. 1 over the dequantized cache
// of Section 3.2), reorganised so that the per-element work is done by the matrix cores:
//
//   scores   sum_d q_d (c_td s_d + z_d) = sum_d (q_d s_d) c_td + sum_d q_d z_d
//   output   sum_t p_t (c_td s_tg + z_tg) = sum_t (p_t s_tg) c_td + sum_t p_t z_tg
//
// The integer codes are the B operand.  Masked into the mantissa of an fp16 with a zero
// exponent field they read as c * 2^-k exactly (k depends on the bit position; differences are
// folded into the A operand), so "conversion" is about one AND per two codes.  The A operand
// carries q_d s_d (scores) or p_t s_tg (output); to keep fp32-class accuracy it is split into a
// high and a low fp16 part held in rows 2j and 2j + 1 of the 16-row tile (j = query head within
// the group, at most 8); a lane of the result tile holds both rows of a head, so the two partial
// results are added in registers after the MFMA.  The zero-point terms: q . z is one more MFMA
// per 32 channels (q and z are exact in fp16), sum_t p_t z_tg is a handful of fp32 FMAs per block.
//
// A work-group owns one (batch, kv head, split) and has two waves: one (the key wave) streams the
// key blocks and produces the softmax numerators of each block, the other (the value wave)
// consumes them one block later and accumulates the output.  The hand-off goes through
// double-buffered LDS tiles and one work-group barrier per block, so score and output work of
// neighbouring blocks overlap on different SIMDs and each wave carries only half of the state
// (which is what lets 4 waves share a SIMD and hide the memory latency).  Each wave writes its
// part of the split's partial result itself; the splits are merged by combine_splits.
#include <hip/hip_ext.h>

#include "kvq_internal.h"

namespace kvq {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

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

// B operand of MFMA m (8 codes of this lane) straight from the packed dwords.  Each code is
// masked into the mantissa of an fp16 whose exponent field is zero: a subnormal number, which
// the matrix core takes at face value, so element e of the operand is exactly
// code * 2^-CodeShift<BITS> * code_weight<BITS>(e) and "conversion" costs about one AND per two
// codes.  (The sum of a tile is aligned to the largest nominal exponent and keeps about 24 bits
// below it, the same as for a normal operand 1 + code * 2^-10, without a "1 +" to remove.)

// log2 of the divisor of the code in the base position: operand element = code * 2^-CodeShift
template <int BITS> struct CodeShift { static constexpr int value = 24; };

// one 32-token block of quantized keys / values as loaded by this lane
template <int BITS>
struct CodeRegs {
    u32x4 q[BITS < 16 ? BITS / 2 : 1];       // the lane's 64 codes, 16 bytes per load
    u32x2 s2;                                // two fp32 scales.  keys: channels 2*lane, +1; values: group lane>>4, tokens 2*(lane&15), +1
    uint32_t s1;                             // the same two scales as an fp16 pair (narrow metadata)
    uint32_t z;                              // zero-points of the same two elements, fp16 pair
    __device__ __forceinline__ uint32_t dw(int k) const { return q[k >> 2][k & 3]; }
};

template <int BITS>
__device__ __forceinline__ half8 codes_operand(const CodeRegs<BITS> &r, int m)
{
    if constexpr (BITS == 8) {
        // bytes (b0, b1), (b2, b3) -> halves 0x0000 | b : b * 2^-24
        const uint32_t w0 = r.dw(2 * m), w1 = r.dw(2 * m + 1);
        return as_half8(__builtin_amdgcn_perm(0u, w0, 0x0C010C00u), __builtin_amdgcn_perm(0u, w0, 0x0C030C02u),
                        __builtin_amdgcn_perm(0u, w1, 0x0C010C00u), __builtin_amdgcn_perm(0u, w1, 0x0C030C02u));
    } else if constexpr (BITS == 4) {
        // nibbles (k, k + 4) of the dword form a pair; mantissa bits 3:0 read c * 2^-24, bits 7:4 read 16 c * 2^-24
        const uint32_t x = r.dw(m), y = x >> 8;
        return as_half8(x & 0x000F000Fu, x & 0x00F000F0u, y & 0x000F000Fu, y & 0x00F000F0u);
    } else {
        // the four 2-bit fields of a byte pair are masked where they sit: mantissa bits 1:0, 3:2, 5:4, 7:6 read
        // c, 4 c, 16 c, 64 c (* 2^-24); the upper byte pair of the dword comes down with one shift
        const uint32_t x = (m & 1) ? r.dw(m >> 1) >> 8 : r.dw(m >> 1);
        return as_half8(x & 0x00030003u, x & 0x000C000Cu, x & 0x00300030u, x & 0x00C000C0u);
    }
}

// power of two by which the A operand must be divided for element e (its code sits higher in
// the mantissa than the base position)
template <int BITS>
__device__ __forceinline__ float code_weight_inv(int e)
{
    if (BITS == 4) return ((e >> 1) & 1) ? 0.0625f : 1.0f;
    if (BITS == 2) return 1.0f / (float)(1 << (2 * ((e >> 1) & 3)));
    return 1.0f;
}

// split two fp32 values into fp16 high parts and fp16 low parts (hi + lo = r to about 2^-21; the
// operands are kept near the top of the fp16 range, so the low parts are normal numbers too)
__device__ __forceinline__ void split_pair(float r0, float r1, uint32_t &hi, uint32_t &lo)
{
    const half2v h = __builtin_bit_cast(half2v, __builtin_amdgcn_cvt_pkrtz(r0, r1));
    const float d0 = r0 - (float)h[0], d1 = r1 - (float)h[1];
    hi = __builtin_bit_cast(uint32_t, h);
    lo = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(d0, d1));
}

// The same for two products a0 b0, a1 b1 whose factors are also at hand rounded to fp16 (a16, b16: pairs).  The
// high parts are the packed fp16 product of the rounded factors (one instruction for both; off the true product by
// less than 2^-9 of it), the low parts what is missing from the true products, each one mixed-precision
// multiply-add.  hi + lo = a b to about 2^-20: four instructions instead of six.
__device__ __forceinline__ void split_products(float a0, float b0, float a1, float b1, uint32_t a16, uint32_t b16,
                                               uint32_t &hi, uint32_t &lo)
{
    const half2v h = __builtin_bit_cast(half2v, a16) * __builtin_bit_cast(half2v, b16);
    const float d0 = __builtin_fmaf(a0, b0, -(float)h[0]), d1 = __builtin_fmaf(a1, b1, -(float)h[1]);
    hi = __builtin_bit_cast(uint32_t, h);
    lo = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(d0, d1));
}

// The packed blocks of one tensor of one (batch, kv head) cache, addressed through buffer resources: a load's address
// is resource base + scalar byte offset of the block + a per-lane offset that never changes, so no vector register
// holds an address.
//
// The block loads of the streaming loop are issued and awaited by hand (issue_block / await_block).  The loop keeps
// one or two blocks in flight behind the one it works on, and what it must wait for is exactly "all but the loads of
// the younger blocks".  Left to the compiler, the wait counts of a loop whose loads stay in flight across the back
// edge came out far too low (all but one to three loads instead of all but eight to ten), the registers of the stage
// about to be loaded were re-used for address arithmetic, which added waits in front of the issue, and a one-word
// load per block was converted to a scalar where it was issued: every iteration cost one full memory round trip.
// The compiler does not know that these loads exist: its own waits (for loads it knows of) can only come out longer
// than needed, never shorter, and the registers a load writes are tied to the asm statements as read-write operands
// from the issue to the wait, so nothing else is put into them in between.
typedef int i32x4 __attribute__((ext_vector_type(4)));

struct BlockStream {
    i32x4 code, meta;                        // buffer resources: base, no stride, no bounds, 32-bit raw format
    i32x4 bexp;                              // exponent words of this cache only (reads beyond it return zero)
    uint32_t l16, l8, l4;                    // this lane's byte offsets into 16-, 8- and 4-byte-per-lane pieces
};

// The loop issues its loads unconditionally (so that the number of loads behind a block is a constant); past the end of
// the group's range they go through a resource with no bytes in range: every load through it is out of range, touches
// no memory and returns zero.
// r, or r with no bytes in range: one scalar select
__device__ __forceinline__ i32x4 pick(bool real, const i32x4 &r)
{
    return i32x4{r[0], r[1], real ? r[2] : 0, r[3]};
}

__device__ __forceinline__ i32x4 buffer_words(const void *base, int bytes = 0x7fffffff)
{
    const uint64_t v = reinterpret_cast<uint64_t>(base);
    return i32x4{__builtin_amdgcn_readfirstlane((int)(uint32_t)v), __builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32) & 0xffff),
                 bytes, 0x00020000};
}

// streams of the keys (values = false) or values of the cache whose first block is number blk0 of the layer
__device__ __forceinline__ BlockStream block_stream(const LayerView &lv, bool values, size_t blk0, int n_cache_blocks, int lane, bool narrow)
{
    BlockStream S;
    const int bits = values ? lv.vbits : lv.kbits;
    S.code = buffer_words((values ? lv.vcode : lv.kcode) + blk0 * block_code_bytes(bits));
    S.meta = buffer_words((values ? lv.vmeta : lv.kmeta) + blk0 * meta_words(narrow));
    S.bexp = buffer_words(lv.bexp + blk0, n_cache_blocks * 4);
    S.l4 = (uint32_t)lane * 4u; S.l8 = (uint32_t)lane * 8u; S.l16 = (uint32_t)lane * 16u;
    return S;
}

// The exponent words (largest key scale / largest value scale of a block, see the quantize kernel) of the blocks that
// kChunk consecutive steps of the sweep visit, one per lane.  A block's word is read from the register with a lane
// index, so the block pipeline holds no load whose result a scalar computation waits for.  Loaded once per chunk of
// the sweep (issued by hand like the block loads; the first one ahead of the first blocks, later ones with a full
// wait, once per kChunk blocks).  Lanes whose block lies beyond the cache read zero.
constexpr int kChunk = 48;                   // steps per chunk: a multiple of both stage counts and of kZChunk, at most 64
constexpr int kZChunk = 16;                  // steps whose zero-point terms of the scores are formed at once (the columns of one tile)

// voff: byte offset of this lane's word in the cache's exponent array
__device__ __forceinline__ void issue_exponents(uint32_t &words, const BlockStream &S, uint32_t voff)
{
    asm volatile("buffer_load_dword %0, %1, %2, 0 offen" : "+v"(words) : "v"(voff), "s"(S.bexp));
}
template <int N>
__device__ __forceinline__ void await_exponents(uint32_t &words)
{
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(words) : "n"(N));
}

// loads of one block per lane
template <int BITS, bool LOADZ = true> constexpr int block_loads() { return BITS < 16 ? BITS / 2 + (LOADZ ? 2 : 1) : 0; }

// Issue the loads of block `blk` of the cache (counted from the cache's first block) into r.  NARROW: the block's
// scales are stored as fp16 (and were used that way by the encoder).  Codes and metadata are read once per call and
// never again before the whole cache has streamed by: the loads carry the non-temporal hint, so the lines are not
// kept in the caches at the expense of anything else (measured: 2-7 % shorter calls, most for the 8-bit pair).
// LOADZ = false: without the zero-points (the key wave fetches those of sixteen blocks at a time, issue_zero_points).
template <int BITS, bool NARROW, bool LOADZ = true>
__device__ __forceinline__ void issue_block(const BlockStream &S0, bool real, int blk, CodeRegs<BITS> &r)
{
    static_assert(BITS < 16, "packed blocks only");
    struct { i32x4 code, meta; uint32_t l16, l8, l4; } S = {pick(real, S0.code), pick(real, S0.meta), S0.l16, S0.l8, S0.l4};
    const int coff = blk * block_code_bytes(BITS), moff = blk * 4 * meta_words(NARROW);
    asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen nt" : "+v"(r.q[0]) : "v"(S.l16), "s"(S.code), "s"(coff));
    if constexpr (BITS >= 4) asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen offset:1024 nt" : "+v"(r.q[BITS >= 4 ? 1 : 0]) : "v"(S.l16), "s"(S.code), "s"(coff));
    if constexpr (BITS == 8) {
        asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen offset:2048 nt" : "+v"(r.q[BITS == 8 ? 2 : 0]) : "v"(S.l16), "s"(S.code), "s"(coff));
        asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen offset:3072 nt" : "+v"(r.q[BITS == 8 ? 3 : 0]) : "v"(S.l16), "s"(S.code), "s"(coff));
    }
    if constexpr (NARROW) {
        asm volatile("buffer_load_dword %0, %1, %2, %3 offen nt" : "+v"(r.s1) : "v"(S.l4), "s"(S.meta), "s"(moff));
        if constexpr (LOADZ) asm volatile("buffer_load_dword %0, %1, %2, %3 offen offset:256 nt" : "+v"(r.z) : "v"(S.l4), "s"(S.meta), "s"(moff));
    } else {
        asm volatile("buffer_load_dwordx2 %0, %1, %2, %3 offen nt" : "+v"(r.s2) : "v"(S.l8), "s"(S.meta), "s"(moff));
        if constexpr (LOADZ) asm volatile("buffer_load_dword %0, %1, %2, %3 offen offset:512 nt" : "+v"(r.z) : "v"(S.l4), "s"(S.meta), "s"(moff));
    }
}

// The zero-points of the keys of kZChunk blocks, fetched as the B operand of one matrix product: lane (n, rq) gets
// channels 32 cb + 8 rq .. + 7 of the n-th of those blocks (16 bytes per load, cb = 0..3).  voff: byte offset, in the
// cache's metadata, of that block's zero-points plus 16 rq.  Issued by hand like the block loads.
__device__ __forceinline__ void issue_zero_points(u32x4 (&zb)[4], const BlockStream &S, bool real, uint32_t voff)
{
    const i32x4 meta = pick(real, S.meta);
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen nt" : "+v"(zb[0]) : "v"(voff), "s"(meta));
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen offset:64 nt" : "+v"(zb[1]) : "v"(voff), "s"(meta));
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen offset:128 nt" : "+v"(zb[2]) : "v"(voff), "s"(meta));
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen offset:192 nt" : "+v"(zb[3]) : "v"(voff), "s"(meta));
}
template <int N>
__device__ __forceinline__ void await_zero_points(u32x4 (&zb)[4])
{
    asm volatile("s_waitcnt vmcnt(%4)" : "+v"(zb[0]), "+v"(zb[1]), "+v"(zb[2]), "+v"(zb[3]) : "n"(N));
}

// Wait until at most N vector memory operations of this wave are outstanding; r's registers are operands, so every
// use of the block comes after the wait.
template <int N, int BITS>
__device__ __forceinline__ void await_loads(CodeRegs<BITS> &r)
{
    if constexpr (BITS == 8)
        asm volatile("s_waitcnt vmcnt(%7)" : "+v"(r.q[0]), "+v"(r.q[BITS == 8 ? 1 : 0]), "+v"(r.q[BITS == 8 ? 2 : 0]), "+v"(r.q[BITS == 8 ? 3 : 0]), "+v"(r.s2), "+v"(r.s1), "+v"(r.z) : "n"(N));
    else if constexpr (BITS == 4)
        asm volatile("s_waitcnt vmcnt(%5)" : "+v"(r.q[0]), "+v"(r.q[BITS == 4 ? 1 : 0]), "+v"(r.s2), "+v"(r.s1), "+v"(r.z) : "n"(N));
    else
        asm volatile("s_waitcnt vmcnt(%4)" : "+v"(r.q[0]), "+v"(r.s2), "+v"(r.s1), "+v"(r.z) : "n"(N));
}

// Block r is needed; the loads of DEPTH - 1 blocks were issued after its own (real ones or empty ones).
template <int BITS, int DEPTH>
__device__ __forceinline__ void await_block(CodeRegs<BITS> &r)
{
    await_loads<(DEPTH - 1) * block_loads<BITS>(), BITS>(r);
}

// The same wait with one of two counts, N + EXTRA when `more_behind` (EXTRA further loads were issued behind the
// block's own) and N otherwise.  One statement with the branch inside: two statements on two code paths would make
// the compiler merge two versions of registers that loads are still writing.
template <int N, int EXTRA, int BITS>
__device__ __forceinline__ void await_loads_either(CodeRegs<BITS> &r, int more_behind)
{
    static_assert(BITS == 2 || BITS == 4 || BITS == 8, "packed blocks only");
#define KVQ_EITHER "s_cmp_eq_u32 %[mb], 0\n\ts_cbranch_scc1 1f\n\ts_waitcnt vmcnt(%[hi])\n\ts_branch 2f\n1:\n\ts_waitcnt vmcnt(%[lo])\n2:"
    if constexpr (BITS == 8)
        asm volatile(KVQ_EITHER : "+v"(r.q[0]), "+v"(r.q[BITS == 8 ? 1 : 0]), "+v"(r.q[BITS == 8 ? 2 : 0]), "+v"(r.q[BITS == 8 ? 3 : 0]), "+v"(r.s2), "+v"(r.s1), "+v"(r.z)
                     : [mb] "s"(more_behind), [hi] "n"(N + EXTRA), [lo] "n"(N) : "scc");
    else if constexpr (BITS == 4)
        asm volatile(KVQ_EITHER : "+v"(r.q[0]), "+v"(r.q[BITS == 4 ? 1 : 0]), "+v"(r.s2), "+v"(r.s1), "+v"(r.z)
                     : [mb] "s"(more_behind), [hi] "n"(N + EXTRA), [lo] "n"(N) : "scc");
    else
        asm volatile(KVQ_EITHER : "+v"(r.q[0]), "+v"(r.s2), "+v"(r.s1), "+v"(r.z)
                     : [mb] "s"(more_behind), [hi] "n"(N + EXTRA), [lo] "n"(N) : "scc");
#undef KVQ_EITHER
}

// a block outside the streaming loop: issue and wait for everything
template <int BITS, bool NARROW>
__device__ __forceinline__ void load_block_now(const BlockStream &S, int blk, CodeRegs<BITS> &r)
{
    issue_block<BITS, NARROW>(S, true, blk, r);
    await_loads<0, BITS>(r);
}

template <int BITS>
__device__ __forceinline__ void clear_regs(CodeRegs<BITS> &r)
{
#pragma unroll
    for (int c = 0; c < (BITS < 16 ? BITS / 2 : 1); c++) r.q[c] = u32x4{0u, 0u, 0u, 0u};
    r.s2 = u32x2{0u, 0u}; r.s1 = 0u; r.z = 0u;
}

// the two scales of a loaded block as floats
template <bool NARROW, int BITS>
__device__ __forceinline__ float2 scales_of(const CodeRegs<BITS> &r)
{
    if constexpr (NARROW) return make_float2(half_lo(r.s1), half_hi(r.s1));
    const uint32_t x = r.s2[0], y = r.s2[1];       // (a bit cast applied to a vector element directly reads element 0)
    return make_float2(__builtin_bit_cast(float, x), __builtin_bit_cast(float, y));
}

// max over the 16 lanes of a DPP row (lanes that share lane >> 4), result in every lane
__device__ __forceinline__ float row_max16(float x)
{
    x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xf, 0xf, false)));   // quad_perm [1,0,3,2]
    x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xf, 0xf, false)));   // quad_perm [2,3,0,1]
    x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xf, 0xf, false)));  // row_half_mirror
    x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xf, 0xf, false)));  // row_mirror
    return x;
}

__device__ __forceinline__ float row_sum16(float x)
{
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xf, 0xf, false));
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xf, 0xf, false));
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xf, 0xf, false));
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xf, 0xf, false));
    return x;
}

// A split's partial results are written through to memory as they are stored (system-scope stores): left in the
// write-back cache they would all be written out at once when the kernel ends, in front of the merge kernel that is
// waiting for it (measured: calls 1-3 % shorter, most with many splits per cache).
__device__ __forceinline__ void store_through(float *p, float2 v)
{
    asm volatile("global_store_dwordx2 %0, %1, off sc0 sc1" ::"v"(p), "v"(v) : "memory");
}

// Work-group barrier that waits for this wave's LDS traffic only: __syncthreads() would also wait for
// the global loads of the next block, which are meant to stay in flight across it.
__device__ __forceinline__ void wg_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// LDS of one key-wave / value-wave pair.  A tiles: row 2j = high parts, row 2j + 1 = low parts of head j.
template <int GQ>
struct __attribute__((aligned(16))) PairLds {
    _Float16 Ak[16][kD + 8];       // key wave: score A tiles [row][channel]
    // value wave: output A tiles [channel group][row][token].  A tile is 16 rows of 80 bytes plus 64 bytes: the four
    // lane rows of a wave write the same (row, token pair) of the four tiles at once, and with this distance between
    // the tiles (336 dwords = 16 banks more than a multiple of 64) they fall on four different quarters of the banks
    struct AvTile { _Float16 at[16][32 + 8]; _Float16 pad[32]; } Av[4];
    _Float16 Zk[kD];               // key wave: key zero-points (fp16 as stored); per-token keys: 32 floats of query sums
    float Mk[2][kD];               // key wave, per-token keys: the block's scales and zero-points as [group][token] floats
    // hand-off: softmax numerators of a block per head, double-buffered.  Rows of 40 floats: the four lane rows of
    // the key wave write rows 2 rq + hh at once, 80 dwords apart = four different quarters of the banks
    float P[2][8][32 + 8];
    float Zt[kZChunk][4][2];       // key wave: zero-point terms of the scores of kZChunk blocks, [block][lane row] = heads 2 rq, 2 rq + 1
    float alpha[2][8];             // hand-off: factor by which everything accumulated before the block shrinks
    int rescale[2][2];             // hand-off: non-zero when alpha is not all ones (padded to 16 bytes)
};

template <int GQ>
struct QueryRegs {
    float q2[GQ][2];               // scaled queries for channels 2*lane, 2*lane+1 (for q * s)
    uint32_t q16[GQ];              // the same pair rounded to fp16
    int nvalid;                    // heads of this tile that exist (the A-tile rows of the others stay zero)
    const _Float16 *Aq;            // LDS: exact fp16 queries as an A tile [16][kD + 8] (rows 2j and 2j + 1 = head j)
    float c, alpha_h;              // log2(e)/sqrt(D); weight of the partial scores
    float vw0, vw1;                // bit-position weights of tokens 2n, 2n+1 in the value codes
    float kappa;                   // per-token keys: weight of the partial score sums
    float qs[2][4];                // per-token keys: c * sum of q over channel group g, heads 2*rq, 2*rq + 1
};

template <int GQ>
struct KeyState {
    float m[2], l[2];              // heads 2*rq, 2*rq + 1: reference max (log2 units), partial sum over this lane's tokens
};

template <int GQ>
struct ValueState {
    float4v O[8];                  // un-normalised output tile per 16-channel block (scaled by 2^(14 - ev - shift))
    float oF[GQ][2];               // fp16-row contributions, channels 2*lane, 2*lane+1
    float accz[GQ];                // sum_t p_t z_tg for group rq, tokens 2n, 2n+1
    int ev;                        // largest value-scale exponent so far
};

// Issue priority of this wave for the next block of its sweep: the more blocks it still has in front of it, the higher.
// The arbiter of a SIMD otherwise prefers the wave that was dispatched first, and the waves dispatched later to a SIMD
// ended 4 us behind the first ones (of 28) although all have the same work; with the priority tied to the progress a
// wave that falls behind is served first until it has caught up (the spread between the first and the last tenth of
// the waves to finish went from 6.3 us to 4.3 us).
// The priority is 3 for the first quarter of the sweep (set before it) and drops by one at the steps where another
// quarter of the blocks is done: three scalar compares per step.
struct PrioritySteps { int to2, to1, to0; };
__device__ __forceinline__ PrioritySteps priority_steps(int total)
{
    return PrioritySteps{(total + 3) >> 2, (total + 1) >> 1, (3 * total + 3) >> 2};
}
__device__ __forceinline__ void priority_at_step(int i, const PrioritySteps &t)
{
    if (i == t.to0) __builtin_amdgcn_s_setprio(0);
    else if (i == t.to1) __builtin_amdgcn_s_setprio(1);
    else if (i == t.to2) __builtin_amdgcn_s_setprio(2);
}

// ------------------------------------------------------------------ key wave

// scores of a quantized block: s[th][hh] for head 2*rq + hh, tokens 16*th + n
// ZB: the zero-point terms c * sum_d q_d z_d of heads 2 rq and 2 rq + 1 come ready-made in zc (zero_point_terms) instead
// of from the block's own zero-points.
template <int KB, int GQ, bool NARROW, bool ZB = false>
__device__ __forceinline__ void scores_packed(const CodeRegs<KB> &blk, uint32_t bexp, const QueryRegs<GQ> &Q, PairLds<GQ> &L, int lane,
                                              float (&s)[2][2], float2 zc = make_float2(0.0f, 0.0f))
{
    const int n = lane & 15, rq = lane >> 4;
    // lift the operand to the top of the fp16 range: the largest q*s of the block lands in [2^12, 2^14)
    const int ek = (int)(bexp & 0xffffu) - 32768;
    const float2 sc = scales_of<NARROW>(blk);
    const float ks0 = ldexpf(sc.x, 14 - ek), ks1 = ldexpf(sc.y, 14 - ek);
    const float ah = ldexpf(Q.alpha_h, ek - 14);
    const uint32_t ks16 = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(ks0, ks1));
#pragma unroll
    for (int j = 0; j < GQ; j++) {
        if (j >= 4 && j >= Q.nvalid) continue;           // (a tile of 8 holds at least 5 heads)
        uint32_t hi, lo;
        split_products(Q.q2[j][0], ks0, Q.q2[j][1], ks1, Q.q16[j], ks16, hi, lo);
        *reinterpret_cast<uint32_t *>(&L.Ak[2 * j][2 * lane]) = hi;
        *reinterpret_cast<uint32_t *>(&L.Ak[2 * j + 1][2 * lane]) = lo;
    }
    if constexpr (!ZB) *reinterpret_cast<uint32_t *>(&L.Zk[2 * lane]) = blk.z;
    wave_lds_sync();
    float4v S0 = {0.0f, 0.0f, 0.0f, 0.0f}, S1 = S0, Z = S0;
#pragma unroll
    for (int cb = 0; cb < 4; cb++) {
        const half8 Aop = *reinterpret_cast<const half8 *>(&L.Ak[n][32 * cb + 8 * rq]);
        S0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(Aop, codes_operand<KB>(blk, cb), S0, 0, 0, 0);
        S1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(Aop, codes_operand<KB>(blk, 4 + cb), S1, 0, 0, 0);
        if constexpr (!ZB) {
            const half8 Bz = *reinterpret_cast<const half8 *>(&L.Zk[32 * cb + 8 * rq]);
            Z = __builtin_amdgcn_mfma_f32_16x16x32_f16(*reinterpret_cast<const half8 *>(Q.Aq + n * (kD + 8) + 32 * cb + 8 * rq), Bz, Z, 0, 0, 0);
        }
    }
    // this lane holds rows 4*rq + i: (high, low) of head 2*rq and (high, low) of head 2*rq + 1
#pragma unroll
    for (int hh = 0; hh < 2; hh++) {
        const float zt = ZB ? (hh ? zc.y : zc.x) : Q.c * Z[2 * hh];
        s[0][hh] = fmaf(ah, S0[2 * hh] + S0[2 * hh + 1], zt);
        s[1][hh] = fmaf(ah, S1[2 * hh] + S1[2 * hh + 1], zt);
    }
}

// The zero-point terms c * sum_d q_d z_d of kZChunk blocks at once: the blocks are the columns of one product whose
// A operand is the exact fp16 query tile (rows 2j = 2j + 1 = head j) and whose B operand came straight from memory
// (issue_zero_points).  Lane (n, rq) ends up with the terms of block n for heads 2 rq and 2 rq + 1 and leaves them in
// L.Zt[n][rq], where the lanes of row rq pick them up block by block.
template <int GQ>
__device__ __forceinline__ void zero_point_terms(const u32x4 (&zb)[4], const QueryRegs<GQ> &Q, PairLds<GQ> &L, int lane)
{
    const int n = lane & 15, rq = lane >> 4;
    float4v Z = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int cb = 0; cb < 4; cb++)
        Z = __builtin_amdgcn_mfma_f32_16x16x32_f16(*reinterpret_cast<const half8 *>(Q.Aq + n * (kD + 8) + 32 * cb + 8 * rq),
                                                   as_half8(zb[cb][0], zb[cb][1], zb[cb][2], zb[cb][3]), Z, 0, 0, 0);
    *reinterpret_cast<float2 *>(&L.Zt[n][rq][0]) = make_float2(Q.c * Z[0], Q.c * Z[2]);
}

// Scores of a quantized block whose keys are grouped per token (one (s, z) per token and 32-channel group):
//   sum_d q_d (c_td s_tg + z_tg) = sum_g [ s_tg * sum_{d in g} q_d c_td  +  z_tg * sum_{d in g} q_d ].
// A channel group is exactly the depth of one MFMA, so each MFMA yields one inner sum per (head, token); the
// scale is applied to its result.  The A tile holds the exact fp16 queries (times a power of two and the code
// position weight; rows 2j, the odd rows are not used) and is built once per kernel.
template <int KB, int GQ, bool NARROW>
__device__ __forceinline__ void scores_packed_per_token(const CodeRegs<KB> &blk, const QueryRegs<GQ> &Q, PairLds<GQ> &L, int lane,
                                                        float (&s)[2][2])
{
    const int n = lane & 15, rq = lane >> 4;
    const float2 sc = scales_of<NARROW>(blk);
    *reinterpret_cast<float2 *>(&L.Mk[0][2 * lane]) = make_float2(sc.x * Q.kappa, sc.y * Q.kappa);
    *reinterpret_cast<float2 *>(&L.Mk[1][2 * lane]) = make_float2(half_lo(blk.z), half_hi(blk.z));
    wave_lds_sync();
    s[0][0] = s[0][1] = s[1][0] = s[1][1] = 0.0f;
    const float4v zero = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int cb = 0; cb < 4; cb++) {
        const half8 Aop = *reinterpret_cast<const half8 *>(&L.Ak[n][32 * cb + 8 * rq]);
        const float4v D0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(Aop, codes_operand<KB>(blk, cb), zero, 0, 0, 0);
        const float4v D1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(Aop, codes_operand<KB>(blk, 4 + cb), zero, 0, 0, 0);
        const float s0 = L.Mk[0][32 * cb + n], s1 = L.Mk[0][32 * cb + 16 + n];
        const float z0 = L.Mk[1][32 * cb + n], z1 = L.Mk[1][32 * cb + 16 + n];
#pragma unroll
        for (int hh = 0; hh < 2; hh++) {
            s[0][hh] = fmaf(s0, D0[2 * hh], fmaf(z0, Q.qs[hh][cb], s[0][hh]));
            s[1][hh] = fmaf(s1, D1[2 * hh], fmaf(z1, Q.qs[hh][cb], s[1][hh]));
        }
    }
    wave_lds_sync();          // the metadata tile is rewritten for the next block
}

// scores of up to 32 fp16 rows (16-bit region or window ring); rows 2j and 2j + 1 of the query tile are equal
template <int GQ>
__device__ __forceinline__ void scores_rows(const uint16_t *row0, const uint16_t *row1, int nt, const QueryRegs<GQ> &Q,
                                            int lane, float (&s)[2][2])
{
    const int n = lane & 15, rq = lane >> 4;
    float4v S0 = {0.0f, 0.0f, 0.0f, 0.0f}, S1 = S0;
#pragma unroll
    for (int cb = 0; cb < 4; cb++) {
        uint4 x0 = make_uint4(0, 0, 0, 0), x1 = x0;
        if (n < nt) x0 = *reinterpret_cast<const uint4 *>(row0 + 32 * cb + 8 * rq);
        if (16 + n < nt) x1 = *reinterpret_cast<const uint4 *>(row1 + 32 * cb + 8 * rq);
        const half8 Aop = *reinterpret_cast<const half8 *>(Q.Aq + n * (kD + 8) + 32 * cb + 8 * rq);
        S0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(Aop, as_half8(x0.x, x0.y, x0.z, x0.w), S0, 0, 0, 0);
        S1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(Aop, as_half8(x1.x, x1.y, x1.z, x1.w), S1, 0, 0, 0);
    }
#pragma unroll
    for (int hh = 0; hh < 2; hh++) {
        s[0][hh] = n < nt ? Q.c * S0[2 * hh] : -INFINITY;
        s[1][hh] = 16 + n < nt ? Q.c * S1[2 * hh] : -INFINITY;
    }
}

// Online softmax over the block's 32 scores per head.  Publishes the numerators (L.P[buf]) and the factor
// by which the value wave must shrink what it has accumulated (L.alpha[buf], L.rescale[buf]).
// The reference maximum only has to keep the numerators in range: it is refreshed (exact maximum over
// the block) when some score exceeds it by more than 1, so numerators stay <= 2 and the fp16 output
// operands cannot overflow.  Heads that do not exist see all-zero operands, hence finite values.
template <int GQ>
__device__ __forceinline__ void softmax_publish(const float (&s)[2][2], KeyState<GQ> &W, PairLds<GQ> &L, int buf, int lane)
{
    const int n = lane & 15, rq = lane >> 4;
    const float mx0 = fmaxf(s[0][0], s[1][0]), mx1 = fmaxf(s[0][1], s[1][1]);
    const bool grow = __any((mx0 > W.m[0] + 1.0f) || (mx1 > W.m[1] + 1.0f));
    if (grow) {
        const float mn0 = fmaxf(W.m[0], row_max16(mx0)), mn1 = fmaxf(W.m[1], row_max16(mx1));
        const float a0 = __builtin_amdgcn_exp2f(W.m[0] - mn0), a1 = __builtin_amdgcn_exp2f(W.m[1] - mn1);
        W.l[0] *= a0; W.l[1] *= a1;
        W.m[0] = mn0; W.m[1] = mn1;
        L.alpha[buf][2 * rq] = a0;            // the 16 lanes of a row write the same value
        L.alpha[buf][2 * rq + 1] = a1;
    }
    if (lane == 0) L.rescale[buf][0] = grow ? 1 : 0;
#pragma unroll
    for (int hh = 0; hh < 2; hh++) {
        const float p0 = __builtin_amdgcn_exp2f(s[0][hh] - W.m[hh]), p1 = __builtin_amdgcn_exp2f(s[1][hh] - W.m[hh]);
        W.l[hh] += p0 + p1;
        L.P[buf][2 * rq + hh][n] = p0;
        L.P[buf][2 * rq + hh][16 + n] = p1;
    }
}

// ------------------------------------------------------------------ value wave

// shrink everything accumulated so far if the key wave moved the reference maximum for this block
template <int GQ>
__device__ __forceinline__ void apply_rescale(ValueState<GQ> &W, const PairLds<GQ> &L, int buf, int lane)
{
    const int rq = lane >> 4;
    if (__builtin_amdgcn_readfirstlane(L.rescale[buf][0])) {
        const float2 al = *reinterpret_cast<const float2 *>(&L.alpha[buf][2 * rq]);
#pragma unroll
        for (int cblk = 0; cblk < 8; cblk++) {
            W.O[cblk][0] *= al.x; W.O[cblk][1] *= al.x;
            W.O[cblk][2] *= al.y; W.O[cblk][3] *= al.y;
        }
#pragma unroll
        for (int j = 0; j < GQ; j++) {
            const float aj = L.alpha[buf][j];
            W.oF[j][0] *= aj; W.oF[j][1] *= aj; W.accz[j] *= aj;
        }
    }
}

// output contribution of a quantized block
template <int VB, int GQ, bool NARROW>
__device__ __forceinline__ void output_packed(const CodeRegs<VB> &blk, uint32_t bexp, const QueryRegs<GQ> &Q, ValueState<GQ> &W,
                                              PairLds<GQ> &L, int buf, int lane)
{
    const int n = lane & 15, rq = lane >> 4;
    // keep p*s at the top of the fp16 range; when a block brings a larger scale, re-base the accumulators (exact)
    const int ev = (int)(bexp >> 16) - 32768;
    if (ev > W.ev) {
#pragma unroll
        for (int cblk = 0; cblk < 8; cblk++)
#pragma unroll
            for (int i = 0; i < 4; i++) W.O[cblk][i] = ldexpf(W.O[cblk][i], W.ev - ev);
        W.ev = ev;
    }
    const float2 sc = scales_of<NARROW>(blk);
    const float sv0 = ldexpf(sc.x * Q.vw0, 14 - W.ev), sv1 = ldexpf(sc.y * Q.vw1, 14 - W.ev);
    const uint32_t sv16 = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(sv0, sv1));
#pragma unroll
    for (int j = 0; j < GQ; j++) {
        if (j >= 4 && j >= Q.nvalid) continue;
        const float2 pp = *reinterpret_cast<const float2 *>(&L.P[buf][j][2 * n]);
        uint32_t hi, lo;
        split_products(pp.x, sv0, pp.y, sv1, __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(pp.x, pp.y)), sv16, hi, lo);
        *reinterpret_cast<uint32_t *>(&L.Av[rq].at[2 * j][2 * n]) = hi;
        *reinterpret_cast<uint32_t *>(&L.Av[rq].at[2 * j + 1][2 * n]) = lo;
        W.accz[j] = fmaf(pp.x, half_lo(blk.z), fmaf(pp.y, half_hi(blk.z), W.accz[j]));
    }
    wave_lds_sync();
#pragma unroll
    for (int gd = 0; gd < 4; gd++) {
        const half8 Aop = *reinterpret_cast<const half8 *>(&L.Av[gd].at[n][8 * rq]);
#pragma unroll
        for (int c2 = 0; c2 < 2; c2++) {
            const int cblk = 2 * gd + c2;
            W.O[cblk] = __builtin_amdgcn_mfma_f32_16x16x32_f16(Aop, codes_operand<VB>(blk, cblk), W.O[cblk], 0, 0, 0);
        }
    }
}

// output contribution of nt fp16 rows: lane owns channels 2*lane, 2*lane+1
template <int GQ>
__device__ __forceinline__ void output_rows(const uint16_t *base, int pos0, int nt, int ring, const uint16_t *new_row, int new_pos,
                                            ValueState<GQ> &W, const PairLds<GQ> &L, int buf, int lane)
{
    // eight rows are fetched at a time with independent loads (a token-by-token loop pays one memory latency per token)
    for (int t0 = 0; t0 < nt; t0 += 8) {
        uint32_t x[8];
#pragma unroll
        for (int k = 0; k < 8; k++) {
            const int pos = pos0 + (t0 + k < nt ? t0 + k : t0);        // past the end: a valid row again, not used
            const uint16_t *row = base + (size_t)(ring ? pos % ring : pos) * kD;
            if (new_row && pos == new_pos) row = new_row;              // the token of a fused append is not in the ring yet
            x[k] = *reinterpret_cast<const uint32_t *>(row + 2 * lane);
        }
#pragma unroll
        for (int k = 0; k < 8; k++) {
            if (t0 + k < nt) {
                const float v0 = half_lo(x[k]), v1 = half_hi(x[k]);
#pragma unroll
                for (int j = 0; j < GQ; j++) {
                    const float pj = L.P[buf][j][t0 + k];
                    W.oF[j][0] = fmaf(pj, v0, W.oF[j][0]);
                    W.oF[j][1] = fmaf(pj, v1, W.oF[j][1]);
                }
            }
        }
    }
}

// ------------------------------------------------------------------ kernel

// Waves per SIMD the register allocation must leave room for: the host plans 2048 groups (4 waves per SIMD) for code
// widths up to 8 bits per key + value element and 1024 (2) beyond; the wider instantiations may
// use the registers that fewer resident waves leave free instead of spilling.
template <int KB, int VB> constexpr int resident_waves() { return (KB < 16 && VB < 16) ? (KB + VB <= 8 ? 4 : 2) : 4; }

template <int KB, int VB, int GQ, bool NARROW, bool KPT>
__global__ __launch_bounds__(128, (resident_waves<KB, VB>())) void decode_mfma(DecodeArgs a)
{
    static_assert(GQ == 4 || GQ == 8, "rows 2j and 2j + 1 of a 16-row tile");
    constexpr bool kFast = KB < 16 && VB < 16;
    // register stages of the phase-1 pipelines (blocks in flight per wave = stages - 1)
    // One block in flight behind the one being worked on (measured with exact wait counts, batch 16..32, 8K..32K
    // tokens: two or three blocks behind are 3-5 % slower for 4- and 2-bit codes and no faster for 8-bit ones: the
    // memory system is the queue here, more requests in it only wait longer).
    constexpr int DK = 2, DV = 2;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);     // wave-uniform on purpose: block indices stay scalar
    const int n = lane & 15, rq = lane >> 4;
    const int split = blockIdx.x, bh = blockIdx.y;
    const int b = bh / a.Hkv, h = bh % a.Hkv;
    const int gq_total = a.Hq / a.Hkv;
    const int head0 = blockIdx.z * GQ;
    const int nvalid = gq_total - head0 < GQ ? gq_total - head0 : GQ;
    const size_t qrow0 = (size_t)b * a.Hq + (size_t)h * gq_total + head0;
    // wave 0 / wave 1 take the key / value role in even work-groups and the other way round in odd ones,
    // so that both kinds of wave land on every SIMD
    const bool key_wave = ((wave ^ (split + bh)) & 1) == 0;

    __shared__ PairLds<GQ> L;
    __shared__ __attribute__((aligned(16))) _Float16 aq_lds[16][kD + 8];

    // ---- work of this group: units [u0, u1) = quantized blocks, then chunks of <= 32 fp16 window tokens.
    // Phase 1 covers the fully quantized blocks (only when both tensors are quantized), phase 2 the rest.
    // Unit number it (counted from u0) is handed over through buffer it & 1.
    int u0, u1;
    split_range(a, split, u0, u1);
    const int f1 = kFast ? (u1 < a.n_blocks ? u1 : a.n_blocks) : u0;     // phase 1 = [u0, f1), phase 2 = [f1, u1)
    const int f1c = f1 > u0 ? f1 : u0;
    const int n1 = f1c - u0, n2 = u1 - f1c;
    const size_t blk0 = (size_t)bh * a.NB;       // first block of this cache in the layer's arrays
    // cache block number of the i-th phase-1 unit (0 <= i < n1).
    // Every group starts its sweep at a different place of its range and wraps around: groups advance at the
    // same pace, and with equal phases their addresses would keep falling on the same memory channels.
    const int rot = n1 > 0 ? (int)(((uint32_t)bh * 40503u + (uint32_t)split * 9973u) % (uint32_t)n1) : 0;
    auto blk1 = [&](int i) {
        const int r = i + rot;
        return u0 + (r < n1 ? r : r - n1);
    };
    auto blk1c = [&](int i) { return i < n1 ? blk1(i) : 0; };     // past the range: any number, the load is an empty one
    // byte offset, in the cache's exponent array, of the word this lane holds for the chunk that starts at step c0
    auto exp_offset = [&](int c0) {
        const int i = c0 + lane;
        const int r = i + rot - (i + rot >= n1 ? n1 : 0);
        return (uint32_t)((i < n1 ? u0 + r : a.n_blocks) * 4);     // beyond the range: beyond the array, reads zero
    };

    QueryRegs<GQ> Q;
    Q.nvalid = nvalid;
    Q.c = a.scale_log2e;
    Q.Aq = &aq_lds[0][0];

    if (key_wave) {
        // =========================================================== key wave
        // the loads are issued in the order in which their results are needed: queries, then the first blocks
        uint32_t qw[GQ];
#pragma unroll
        for (int j = 0; j < GQ; j++) {
            qw[j] = 0;
            if (j < nvalid) qw[j] = *reinterpret_cast<const uint32_t *>(a.q + (qrow0 + j) * kD + 2 * lane);
        }
        const BlockStream KS = block_stream(a.lv, false, blk0, a.n_blocks, lane, NARROW);
        uint32_t kexp = 0;                               // exponent words of the chunk's blocks, one per lane
        CodeRegs<KB> kr[DK];
        // per-channel keys: the zero-points do not come with the blocks but for kZChunk blocks at a time, as the operand
        // of one matrix product (zero_point_terms), which saves 4 of the 12 matrix instructions of a block's scores
        // (not next to 8-bit values in a tile of 8 heads: that instantiation has no registers to spare and would spill)
        constexpr bool kZB = kFast && !KPT && !(GQ == 8 && VB == 8);
        constexpr int NLK = block_loads<KB, !kZB>();
        u32x4 zb[4];
        // byte offset, in the cache's metadata, of the 16 bytes of zero-points this lane fetches for the chunk of steps
        // that starts at z0 (beyond the range: those of some block of the range, not used)
        auto zero_point_offset = [&](int z0) {
            const int i = z0 + n;
            return (uint32_t)(blk1c(i) * (4 * meta_words(NARROW)) + (NARROW ? 256 : 512) + 16 * rq);
        };
        if constexpr (kFast) {
#pragma unroll
            for (int d = 0; d < DK; d++) clear_regs(kr[d]);
            issue_exponents(kexp, KS, exp_offset(0));
            if constexpr (kZB) {
#pragma unroll
                for (int cb = 0; cb < 4; cb++) zb[cb] = u32x4{0u, 0u, 0u, 0u};
                issue_zero_points(zb, KS, n1 > 0, zero_point_offset(0));
            }
#pragma unroll
            for (int d = 0; d < DK - 1; d++) issue_block<KB, NARROW, !kZB>(KS, d < n1, blk1c(d), kr[d]);
        }
        {
            // queries divided by a power of two that brings the largest to [0.5, 1).  Per-channel keys: with the softmax
            // constant folded in, for the q * s operand.  Per-token keys: the raw fp16 queries, scaled exactly.
            constexpr bool kPerToken = KPT && KB < 16;
            float qraw[GQ][2];
            float qmax = 0.0f;
#pragma unroll
            for (int j = 0; j < GQ; j++) {
                const uint32_t w = qw[j];
                qraw[j][0] = kPerToken ? half_lo(w) : half_lo(w) * Q.c;
                qraw[j][1] = kPerToken ? half_hi(w) : half_hi(w) * Q.c;
                qmax = fmaxf(qmax, fmaxf(fabsf(qraw[j][0]), fabsf(qraw[j][1])));
            }
            // maximum over the wave: 16-lane rows by DPP, the 4 rows as unsigned integers (the values are >= 0)
            const int qrow = __builtin_bit_cast(int, row_max16(qmax));
            uint32_t qbits = (uint32_t)__builtin_amdgcn_readlane(qrow, 0);
#pragma unroll
            for (int r = 1; r < 4; r++) {
                const uint32_t o = (uint32_t)__builtin_amdgcn_readlane(qrow, 16 * r);
                qbits = o > qbits ? o : qbits;
            }
            qmax = __builtin_bit_cast(float, qbits);
            int qexp = 0;
            if (qmax > 0.0f) (void)frexpf(qmax, &qexp);      // qmax = f * 2^qexp, f in [0.5, 1)
            constexpr int kshift = CodeShift<KB < 16 ? KB : 8>::value;
            const float w0 = code_weight_inv<KB < 16 ? KB : 8>((2 * lane) & 7), w1 = code_weight_inv<KB < 16 ? KB : 8>((2 * lane + 1) & 7);
            if constexpr (kPerToken) {
                // constant A tile: row 2j = q_j * 2^(13 - qexp) / (code position weight), exact in fp16; odd rows unused
                Q.kappa = Q.c * ldexpf(1.0f, kshift + qexp - 13);
                float *qs_lds = reinterpret_cast<float *>(&L.Zk[0]);      // [head][group] sums, 4 * GQ <= 32 floats
#pragma unroll
                for (int j = 0; j < GQ; j++) {
                    *reinterpret_cast<uint32_t *>(&L.Ak[2 * j][2 * lane]) =
                        __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(ldexpf(qraw[j][0], 13 - qexp) * w0, ldexpf(qraw[j][1], 13 - qexp) * w1));
                    *reinterpret_cast<uint32_t *>(&L.Ak[2 * j + 1][2 * lane]) = 0u;
                    const float part = row_sum16(qraw[j][0] + qraw[j][1]);       // this lane row's channel group is rq
                    if (n == 0) qs_lds[4 * j + rq] = part * Q.c;
                }
                wave_lds_sync();
#pragma unroll
                for (int hh = 0; hh < 2; hh++)
#pragma unroll
                    for (int g = 0; g < 4; g++) Q.qs[hh][g] = 2 * rq + hh < nvalid ? qs_lds[4 * ((2 * rq + hh) % GQ) + g] : 0.0f;
            } else {
                Q.alpha_h = ldexpf(1.0f, kshift + qexp);     // undo the code position and 2^-qexp of q
#pragma unroll
                for (int j = 0; j < GQ; j++) {
                    Q.q2[j][0] = ldexpf(qraw[j][0], -qexp) * w0;
                    Q.q2[j][1] = ldexpf(qraw[j][1], -qexp) * w1;
                    Q.q16[j] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(Q.q2[j][0], Q.q2[j][1]));
                }
            }
            {
                // A-tile rows of heads that do not exist are never written: they must read as zero
                const int row0 = 2 * (GQ == 8 ? nvalid : GQ);
                for (int i = lane; i < (16 - row0) * (kD + 8) / 8; i += 64)
                    reinterpret_cast<uint4 *>(&L.Ak[row0][0])[i] = make_uint4(0, 0, 0, 0);
            }
        }
        wg_barrier();                                   // the value wave has written the exact-fp16 query tile
        KeyState<GQ> W;
#pragma unroll
        for (int i = 0; i < 2; i++) { W.m[i] = -INFINITY; W.l[i] = 0.0f; }
        float s[2][2];
        if constexpr (kFast) {
            // DK register stages in rotation: stage d is consumed while the loads of the next DK - 1 units (as far as
            // there are any) are in flight.
            // The sweep goes in chunks of kChunk steps (one register of exponent words each); a chunk starts at stage 0.
            await_exponents<(DK - 1) * NLK>(kexp);                         // the first chunk's: issued ahead of the first blocks
            const PrioritySteps prio = priority_steps(n1);
            if (n1 > 0) __builtin_amdgcn_s_setprio(3);
            for (int c0 = 0; c0 < n1; c0 += kChunk) {
                if (c0 > 0) {
                    issue_exponents(kexp, KS, exp_offset(c0));
                    await_exponents<0>(kexp);
                }
                const int cend = c0 + kChunk < n1 ? c0 + kChunk : n1;
                for (int z0 = c0; z0 < cend; z0 += kZChunk) {
                    const int zend = z0 + kZChunk < cend ? z0 + kZChunk : cend;
                    if constexpr (kZB) {
                        // The chunk's zero-points were asked for a chunk ago (the first chunk's ahead of the first
                        // blocks): they are older than every load still allowed to be pending here.  Form the chunk's
                        // terms, then ask for the next chunk's; those four loads go out in front of the first step's
                        // block loads, so that step alone waits with four more loads allowed behind its block.
                        await_zero_points<(DK - 1) * NLK>(zb);
                        zero_point_terms<GQ>(zb, Q, L, lane);
                        wave_lds_sync();
                        issue_zero_points(zb, KS, z0 + kZChunk < n1, zero_point_offset(z0 + kZChunk));
                    }
                    bool more = true;
                    for (int i = z0; more;) {
#pragma unroll
                        for (int d = 0; d < DK; d++) {
                            if (more) {
                                priority_at_step(i, prio);
                                issue_block<KB, NARROW, !kZB>(KS, i + DK - 1 < n1, blk1c(i + DK - 1), kr[(d + DK - 1) % DK]);
                                if constexpr (kZB) await_loads_either<(DK - 1) * NLK, 4, KB>(kr[d], __builtin_amdgcn_readfirstlane(i == z0 ? 1 : 0));
                                else await_block<KB, DK>(kr[d]);
                                const uint32_t ew = (uint32_t)__builtin_amdgcn_readlane((int)kexp, i - c0);
                                if constexpr (KPT) scores_packed_per_token<KB, GQ, NARROW>(kr[d], Q, L, lane, s);
                                else if constexpr (kZB)
                                    scores_packed<KB, GQ, NARROW, true>(kr[d], ew, Q, L, lane, s, *reinterpret_cast<const float2 *>(&L.Zt[i - z0][rq][0]));
                                else scores_packed<KB, GQ, NARROW>(kr[d], ew, Q, L, lane, s);
                                softmax_publish<GQ>(s, W, L, i & 1, lane);
                                wg_barrier();
                                more = ++i < zend;
                            }
                        }
                    }
                }
            }
            __builtin_amdgcn_s_setprio(0);
#pragma unroll
            for (int d = 0; d < DK; d++) await_loads<0, KB>(kr[d]);      // the empty loads past the end of the range, before
            await_exponents<0>(kexp);                                    // their registers go back to the compiler
            if constexpr (kZB) await_zero_points<0>(zb);
        }
        for (int i = 0; i < n2; i++) {
            const int u = f1c + i;
            const bool packed = u < a.n_blocks;
            const int pos0 = packed ? u * kG : a.n_blocks * kG + (u - a.n_blocks) * 32;
            const int nt = packed ? 32 : (a.n_res - (u - a.n_blocks) * 32 < 32 ? a.n_res - (u - a.n_blocks) * 32 : 32);
            bool k_rows = true;
            if constexpr (KB < 16) if (packed) {
                k_rows = false;
                CodeRegs<KB> r;
                clear_regs(r);
                load_block_now<KB, NARROW>(KS, u, r);
                if constexpr (KPT) scores_packed_per_token<KB, GQ, NARROW>(r, Q, L, lane, s);
                else scores_packed<KB, GQ, NARROW>(r, a.lv.bexp[blk0 + u], Q, L, lane, s);
            }
            if (k_rows) {
                const uint16_t *kbase = packed ? reinterpret_cast<const uint16_t *>(a.lv.kcode) + (size_t)bh * a.NB * kG * kD
                                               : a.lv.kres + (size_t)bh * a.RC * kD;
                const int p0 = pos0 + n, p1 = pos0 + 16 + n;
                const uint16_t *row0 = kbase + (size_t)(packed ? p0 : p0 % a.RC) * kD, *row1 = kbase + (size_t)(packed ? p1 : p1 % a.RC) * kD;
                if (!packed && a.k_new && a.new_pos >= pos0 && a.new_pos < pos0 + nt) {
                    // fused append: this chunk holds the new token.  Read its row from the caller's tensor and
                    // put it into the window ring for later launches (nothing reads that slot in this launch).
                    const uint16_t *src = a.k_new + (size_t)bh * kD;
                    if (p0 == a.new_pos) row0 = src;
                    if (p1 == a.new_pos) row1 = src;
                    reinterpret_cast<uint32_t *>(a.lv.kres + ((size_t)bh * a.RC + a.new_pos % a.RC) * kD)[lane] = reinterpret_cast<const uint32_t *>(src)[lane];
                }
                scores_rows<GQ>(row0, row1, nt, Q, lane, s);
            }
            softmax_publish<GQ>(s, W, L, (n1 + i) & 1, lane);
            wg_barrier();
        }
        wg_barrier();                                   // the value wave consumes the last unit
        // ---- result of the key wave: reference max and sum per head
#pragma unroll
        for (int hh = 0; hh < 2; hh++) {
            const float lsum = row_sum16(W.l[hh]);
            const int j = 2 * rq + hh;
            if (n == 0 && j < nvalid) {
                const size_t prow = (qrow0 + j) * a.splits + split;
                store_through(a.part_ml + prow * 2, make_float2(W.m[hh], lsum));
            }
        }
    } else {
        // =========================================================== value wave (one unit behind the key wave)
        // rows 2j and 2j + 1 of the exact-fp16 query tile (16 rows x 256 bytes); rows of absent heads are zero.
        // The loads are issued in the order in which their results are needed: queries, then the first blocks.
        uint4 qx[4];
#pragma unroll
        for (int pass = 0; pass < 4; pass++) {
            const int jr = (4 * pass + rq) >> 1;
            qx[pass] = make_uint4(0, 0, 0, 0);
            if (jr < nvalid) qx[pass] = *reinterpret_cast<const uint4 *>(a.q + (qrow0 + jr) * kD + 8 * n);
        }
        const BlockStream VS = block_stream(a.lv, true, blk0, a.n_blocks, lane, NARROW);
        uint32_t vexp = 0;
        CodeRegs<VB> vr[DV];
        if constexpr (kFast) {
#pragma unroll
            for (int d = 0; d < DV; d++) clear_regs(vr[d]);
            issue_exponents(vexp, VS, exp_offset(0));
#pragma unroll
            for (int d = 0; d < DV - 1; d++) issue_block<VB, NARROW>(VS, d < n1, blk1c(d), vr[d]);
        }
#pragma unroll
        for (int pass = 0; pass < 4; pass++) *reinterpret_cast<uint4 *>(&aq_lds[4 * pass + rq][8 * n]) = qx[pass];
        {
            const int row0 = 2 * (GQ == 8 ? nvalid : GQ);
            const int per = (16 - row0) * (32 + 8) / 8;              // 16-byte pieces of the unused rows per channel group
            for (int i = lane; i < 4 * per; i += 64)
                reinterpret_cast<uint4 *>(&L.Av[i / per].at[row0][0])[i % per] = make_uint4(0, 0, 0, 0);
        }
        Q.vw0 = code_weight_inv<VB < 16 ? VB : 8>((2 * n) & 7);
        Q.vw1 = code_weight_inv<VB < 16 ? VB : 8>((2 * n + 1) & 7);
        wg_barrier();                                   // query tile handed to the key wave
        ValueState<GQ> W;
#pragma unroll
        for (int cblk = 0; cblk < 8; cblk++) W.O[cblk] = float4v{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int j = 0; j < GQ; j++) { W.oF[j][0] = W.oF[j][1] = 0.0f; W.accz[j] = 0.0f; }
        W.ev = -100;
        wg_barrier();                                   // the key wave has produced the first unit
        if constexpr (kFast) {
            await_exponents<(DV - 1) * block_loads<VB>()>(vexp);
            const PrioritySteps prio = priority_steps(n1);
            if (n1 > 0) __builtin_amdgcn_s_setprio(3);
            for (int c0 = 0; c0 < n1; c0 += kChunk) {
                if (c0 > 0) {
                    issue_exponents(vexp, VS, exp_offset(c0));
                    await_exponents<0>(vexp);
                }
                const int cend = c0 + kChunk < n1 ? c0 + kChunk : n1;
                bool more = true;
                for (int i = c0; more;) {
#pragma unroll
                    for (int d = 0; d < DV; d++) {
                        if (more) {
                            priority_at_step(i, prio);
                            issue_block<VB, NARROW>(VS, i + DV - 1 < n1, blk1c(i + DV - 1), vr[(d + DV - 1) % DV]);
                            await_block<VB, DV>(vr[d]);
                            const uint32_t ew = (uint32_t)__builtin_amdgcn_readlane((int)vexp, i - c0);
                            // (always true here; as a run-time test it keeps the rarely taken re-base and rescale
                            // paths out of line, without it the register count of the loop grows by half)
                            if (i < n1) {
                                apply_rescale<GQ>(W, L, i & 1, lane);
                                output_packed<VB, GQ, NARROW>(vr[d], ew, Q, W, L, i & 1, lane);
                            }
                            wg_barrier();
                            more = ++i < cend;
                        }
                    }
                }
            }
            __builtin_amdgcn_s_setprio(0);
#pragma unroll
            for (int d = 0; d < DV; d++) await_loads<0, VB>(vr[d]);
            await_exponents<0>(vexp);
        }
        for (int i = 0; i < n2; i++) {
            const int u = f1c + i, buf = (n1 + i) & 1;
            const bool packed = u < a.n_blocks;
            const int pos0 = packed ? u * kG : a.n_blocks * kG + (u - a.n_blocks) * 32;
            const int nt = packed ? 32 : (a.n_res - (u - a.n_blocks) * 32 < 32 ? a.n_res - (u - a.n_blocks) * 32 : 32);
            apply_rescale<GQ>(W, L, buf, lane);
            bool v_rows = true;
            if constexpr (VB < 16) if (packed) {
                v_rows = false;
                CodeRegs<VB> r;
                clear_regs(r);
                load_block_now<VB, NARROW>(VS, u, r);
                output_packed<VB, GQ, NARROW>(r, a.lv.bexp[blk0 + u], Q, W, L, buf, lane);
            }
            if (v_rows) {
                const uint16_t *vbase = packed ? reinterpret_cast<const uint16_t *>(a.lv.vcode) + (size_t)bh * a.NB * kG * kD
                                               : a.lv.vres + (size_t)bh * a.RC * kD;
                const uint16_t *new_row = nullptr;
                if (!packed && a.v_new && a.new_pos >= pos0 && a.new_pos < pos0 + nt) {
                    new_row = a.v_new + (size_t)bh * kD;
                    reinterpret_cast<uint32_t *>(a.lv.vres + ((size_t)bh * a.RC + a.new_pos % a.RC) * kD)[lane] = reinterpret_cast<const uint32_t *>(new_row)[lane];
                }
                output_rows<GQ>(vbase, pos0, nt, packed ? 0 : a.RC, new_row, a.new_pos, W, L, buf, lane);
            }
            wg_barrier();
        }
        // ---- result of the value wave: un-normalised output per head and channel.  The tile layout (lane =
        // channel 16 cblk + n, rows of heads 2 rq, 2 rq + 1) is turned into (lane = channels 2 lane, 2 lane + 1,
        // all heads) through the A-tile memory, which is no longer needed.
        static_assert(sizeof(L.Av) >= GQ * kD * sizeof(float), "output staging fits the A tiles");
        float *o_lds = reinterpret_cast<float *>(&L.Av[0].at[0][0]);
        constexpr int vshift = CodeShift<VB < 16 ? VB : 8>::value;
        const float wO = ldexpf(1.0f, vshift + W.ev - 14);       // high and low parts carry the same weight
        wave_lds_sync();
#pragma unroll
        for (int hh = 0; hh < 2; hh++) {
            const int j = 2 * rq + hh;
            if (j < GQ) {
#pragma unroll
                for (int cblk = 0; cblk < 8; cblk++) o_lds[j * kD + 16 * cblk + n] = wO * (W.O[cblk][2 * hh] + W.O[cblk][2 * hh + 1]);
            }
        }
        wave_lds_sync();
#pragma unroll
        for (int j = 0; j < GQ; j++) {
            // sum_t p_t z_tg of this lane's channel group (lane >> 4), over the 16 lanes that hold its tokens
            const float az = row_sum16(W.accz[j]);
            if (j < nvalid) {
                const float2 t = *reinterpret_cast<const float2 *>(&o_lds[j * kD + 2 * lane]);
                const size_t prow = (qrow0 + j) * a.splits + split;
                store_through(a.part_o + prow * kD + 2 * lane, make_float2(t.x + W.oF[j][0] + az, t.y + W.oF[j][1] + az));
            }
        }
    }
}

struct LaunchEvents { hipEvent_t begin, end; };

template <int KB, int VB, bool NARROW, bool KPT>
hipError_t launch_gq(const DecodeArgs &a, hipStream_t s, LaunchEvents ev)
{
    const int gq = a.Hq / a.Hkv;
    const int BH = a.B * a.Hkv;
    const dim3 block(128);
    const dim3 grid(a.splits, BH, gq <= 4 ? 1 : (gq + 7) / 8);
    if (ev.begin && ev.end) {
        // measurement: the runtime's extended launch stamps the events with the dispatch's own start and end times
        if (gq <= 4) hipExtLaunchKernelGGL((decode_mfma<KB, VB, 4, NARROW, KPT>), grid, block, 0, s, ev.begin, ev.end, 0, a);
        else hipExtLaunchKernelGGL((decode_mfma<KB, VB, 8, NARROW, KPT>), grid, block, 0, s, ev.begin, ev.end, 0, a);
    } else if (gq <= 4) {
        hipLaunchKernelGGL((decode_mfma<KB, VB, 4, NARROW, KPT>), grid, block, 0, s, a);
    } else {
        hipLaunchKernelGGL((decode_mfma<KB, VB, 8, NARROW, KPT>), grid, block, 0, s, a);
    }
    return hipGetLastError();
}

template <int KB, bool NARROW, bool KPT>
hipError_t launch_vb(const DecodeArgs &a, hipStream_t s, LaunchEvents ev)
{
    switch (a.lv.vbits) {
    case 2: return launch_gq<KB, 2, NARROW, KPT>(a, s, ev);
    case 4: return launch_gq<KB, 4, NARROW, KPT>(a, s, ev);
    case 8: return launch_gq<KB, 8, NARROW, KPT>(a, s, ev);
    default: return launch_gq<KB, 16, NARROW, KPT>(a, s, ev);
    }
}

template <bool NARROW>
hipError_t launch_kb(const DecodeArgs &a, hipStream_t s, LaunchEvents ev)
{
    // the key grouping only matters for quantized keys
    if (a.lv.kpt) {
        switch (a.lv.kbits) {
        case 2: return launch_vb<2, NARROW, true>(a, s, ev);
        case 4: return launch_vb<4, NARROW, true>(a, s, ev);
        case 8: return launch_vb<8, NARROW, true>(a, s, ev);
        default: break;
        }
    }
    switch (a.lv.kbits) {
    case 2: return launch_vb<2, NARROW, false>(a, s, ev);
    case 4: return launch_vb<4, NARROW, false>(a, s, ev);
    case 8: return launch_vb<8, NARROW, false>(a, s, ev);
    default: return launch_vb<16, NARROW, false>(a, s, ev);
    }
}

}  // namespace

hipError_t launch_decode_mfma(const DecodeArgs &a, hipStream_t s, hipEvent_t ev_begin, hipEvent_t ev_end)
{
    if (a.B * a.Hkv > 65535) return hipErrorInvalidConfiguration;
    const LaunchEvents ev = {ev_begin, ev_end};
    return a.lv.narrow ? launch_kb<true>(a, s, ev) : launch_kb<false>(a, s, ev);
}

}  // namespace kvq
