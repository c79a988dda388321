// Internal declarations shared by the host API and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvq_layout.h"

namespace kvq {

// Device pointers of one layer's cache inside the workspace.
struct LayerView {
    uint8_t *kcode;       // [BH][NB] blocks of block_code_bytes(kbits)
    float *kmeta;         // [BH][NB] metadata blocks of meta_words(narrow) dwords (absent when kbits == 16)
    uint8_t *vcode;       // [BH][NB] blocks of block_code_bytes(vbits)
    float *vmeta;         // [BH][NB] metadata blocks of meta_words(narrow) dwords (absent when vbits == 16)
    uint32_t *bexp;       // [BH][NB] binary exponents of the block's largest key / value scale (lo / hi half)
    uint16_t *kres;       // [BH][RC][128] fp16 ring, slot = position % RC
    uint16_t *vres;
    int kbits, vbits;
    int narrow;           // 1: scales stored (and used) as fp16
    int kpt;              // 1: keys grouped per token over 32 channels (metadata laid out like the values')
};

struct QuantArgs {
    LayerView lv;
    const uint16_t *k_in, *v_in;   // fp16 [BH][n_in][128], the tokens of this append
    int n_in;                      // tokens in this append
    int t_old;                     // tokens held before this append
    int first_block;               // first block to write (= old N_p / 32)
    int n_blocks;                  // blocks to write
    int BH;                        // batch * kv heads
    int NB;                        // block capacity per (b, h)
    int RC;                        // ring capacity (R + G)
};

struct ResidualCopyArgs {
    LayerView lv;
    const uint16_t *k_in, *v_in;
    int n_in, t_old;
    int pos0, pos1;                // absolute positions [pos0, pos1) to copy from the input into the ring
    int BH, RC;
};

struct ExportArgs {
    LayerView lv;
    uint8_t *k_codes, *v_codes;
    float *k_scale, *k_zero, *v_scale, *v_zero;
    uint16_t *k_res, *v_res;
    int n_packed, n_res;
    int BH, NB, RC;
};

struct DecodeArgs {
    LayerView lv;
    const uint16_t *q;     // fp16 [B][Hq][128]
    uint16_t *out;         // fp16 [B][Hq][128]
    float *part_o;         // [B*Hq][splits][128] un-normalised partial outputs
    float *part_ml;        // [B*Hq][splits][2]   (running max in log2 units, sum)
    int B, Hq, Hkv;
    int n_blocks;          // quantized blocks (N_p / 32)
    int n_res;             // fp16 tokens at positions [32*n_blocks, 32*n_blocks + n_res)
    int NB, RC;
    int splits;            // gridDim.x
    int units_per_split;   // work units per split: the last split_rem splits take one more.  Units are the quantized blocks, then
    int split_rem;         // (owned by the last split, counted as a few units) the fp16 window
    float scale_log2e;     // log2(e) / sqrt(D)
    // fused append of one token per sequence (matrix-core kernel only): its fp16 rows [B*Hkv][128], not yet in the
    // window ring; the kernel reads them from here and stores them into the ring for later launches.  NULL: none.
    const uint16_t *k_new, *v_new;
    int new_pos;           // absolute position of that token
};

struct PrefillArgs {
    LayerView lv;
    const uint16_t *q;     // fp16 [B][Hq][n_q][128]: the last n_q positions
    uint16_t *out;         // fp16 [B][Hq][n_q][128]
    int B, Hq, Hkv;
    int n_blocks;          // quantized blocks (N_p / 32)
    int n_res;             // fp16 tokens at positions [32*n_blocks, 32*n_blocks + n_res)
    int NB, RC;
    int n_q;               // 1 <= n_q <= 32*n_blocks + n_res
    float scale_log2e;     // log2(e) / sqrt(D)
    // one launch covers the (batch, kv head) caches [bh0, bh0 + n_bh); their packed units are dequantized into
    // scratch[n_bh][n_blocks][prefill_unit_bytes()] first
    uint8_t *scratch;
    int bh0, n_bh;
    // one record of prefill_select_bytes() per cache of the launch (written and read by the launch's kernels): which 32
    // key channels keep the remainders of their fp16 rounding, or that all do
    uint8_t *select;
};

// Work units [u0, u1) of a split: units are the quantized blocks, then the chunks of <= 32 fp16 window tokens.  The
// blocks and the window's weight (a few virtual units behind the blocks) are dealt out evenly: units_per_split each,
// one more for the last split_rem splits (the window's split among them: its share holds the window's units
// first); the last split owns the window and whatever blocks its share leaves room
// for (possibly none).
__device__ __forceinline__ void split_range(const DecodeArgs &a, int split, int &u0, int &u1)
{
    const int first_big = a.splits - a.split_rem;            // the last split_rem splits take one unit more
    u0 = split * a.units_per_split + (split > first_big ? split - first_big : 0);
    u1 = u0 + a.units_per_split + (split >= first_big ? 1 : 0);
    if (u0 > a.n_blocks) u0 = a.n_blocks;
    if (u1 > a.n_blocks) u1 = a.n_blocks;
    if (split == a.splits - 1) u1 = a.n_blocks + (a.n_res + 31) / 32;
}

hipError_t launch_quantize(const QuantArgs &a, hipStream_t s);
hipError_t launch_residual_copy(const ResidualCopyArgs &a, hipStream_t s);
hipError_t launch_export(const ExportArgs &a, hipStream_t s);
hipError_t launch_decode_valu(const DecodeArgs &a, hipStream_t s);
// ev_begin / ev_end (both or neither): receive the start and stop time stamps of the kernel's own dispatch
hipError_t launch_decode_mfma(const DecodeArgs &a, hipStream_t s, hipEvent_t ev_begin = nullptr, hipEvent_t ev_end = nullptr);
size_t prefill_unit_bytes();     // scratch bytes per packed unit (32 tokens) of one (batch, kv head) cache
size_t prefill_select_bytes();   // bytes of the channel-selection record of one (batch, kv head) cache
// decides for the caches [bh0, bh0 + n_bh) which key channels keep their low parts (a.select: their records; layers with
// packed, per-channel quantized keys only); ev_begin (may be null) receives the kernel's start
hipError_t launch_prefill_select(const PrefillArgs &a, hipStream_t s, hipEvent_t ev_begin = nullptr);
// dequantizes the packed units of the caches [bh0, bh0 + n_bh) into the scratch area (a.select: their selection
// records, or null: every channel keeps its low part), then attends; ev_begin / ev_end
// (either may be null) receive the start of the first and the end of the last kernel
hipError_t launch_prefill_attention(const PrefillArgs &a, hipStream_t s, hipEvent_t ev_begin = nullptr, hipEvent_t ev_end = nullptr);
hipError_t launch_combine(const DecodeArgs &a, hipStream_t s);

}  // namespace kvq
