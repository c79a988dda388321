// Host side of the C ABI declared in include/kvq.h: argument validation, workspace
// planning, the per-layer token bookkeeping of the full-precision window, and the
// kernel launches.  No device memory is allocated here and nothing synchronises.
#include "../../include/kvq.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "kvq_internal.h"

namespace {

constexpr int kMaxSplits = 128;
constexpr int kPrefillChunk = 16;   // caches dequantized per prefill-attention pass (two per XCD)
constexpr int kWindowWeight = 6;   // cost of a chunk (<= 32 tokens) of the fp16 window in a split's share, in packed blocks
constexpr size_t kAlign = 256;

thread_local char g_last_error[256] = "";

// Built-in scratch of kvq_decode_attention_noalloc: the partial results of the token-range splits, which the other
// decode calls keep in the caller's workspace.  One record per (query row, split): 128 un-normalised outputs, then
// (further back) the pair (maximum, sum).  Every GPU the library runs on holds its own copy until the process ends.
constexpr size_t kStaticRecords = 16384;                                   // 2048 groups x 8 grouped query heads
constexpr size_t kStaticOutBytes = kStaticRecords * kvq::kD * sizeof(float);
constexpr size_t kStaticBytes = kStaticOutBytes + kStaticRecords * 2 * sizeof(float);      // 8.1 MiB
constexpr int kMaxDevices = 64;
}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {
// device address of `scratch` on each GPU (the array's name is only a host-side handle), looked up once per device
std::atomic<unsigned char *> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

bool bits_ok(int b) { return b == 2 || b == 4 || b == 8 || b == 16; }

bool config_ok(const kvq_config *c)
{
    if (!c || !c->kbits || !c->vbits) return false;
    if (c->n_layers < 1 || c->batch < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1) return false;
    if (c->n_q_heads % c->n_kv_heads) return false;
    if (c->head_dim != kvq::kD || c->group != kvq::kG) return false;
    if (c->max_tokens < 1 || c->residual < 0 || c->residual > (1 << 20)) return false;
    if ((int64_t)c->batch * c->n_q_heads > (1 << 24)) return false;
    if ((int64_t)c->batch * c->n_kv_heads > 65535) return false;        // one grid row per (batch, kv head)
    for (int l = 0; l < c->n_layers; l++)
        if (!bits_ok(c->kbits[l]) || !bits_ok(c->vbits[l])) return false;
    if (c->meta_dtype != KVQ_META_FP32 && c->meta_dtype != KVQ_META_FP16) return false;
    if (c->key_mode != KVQ_KEYS_PER_CHANNEL && c->key_mode != KVQ_KEYS_PER_TOKEN) return false;
    return true;
}

struct LayerPlan {
    size_t kcode, kmeta, vcode, vmeta, bexp, kres, vres;   // byte offsets into the workspace
};

struct Plan {
    std::vector<LayerPlan> layer;
    size_t part_o, part_ml, prefill_scratch, prefill_select, total;
    int NB, RC;
    int prefill_chunk;      // (batch, kv head) caches whose dequantized units the prefill scratch holds at a time
};

Plan make_plan(const kvq_config *c)
{
    Plan p;
    const size_t BH = (size_t)c->batch * c->n_kv_heads;
    p.NB = c->max_tokens / kvq::kG;                 // N_p never exceeds G * floor(max_tokens / G)
    p.RC = c->residual + kvq::kG;                   // the fp16 window never holds R + G tokens or more
    const bool narrow = c->meta_dtype == KVQ_META_FP16;
    size_t off = 0;
    p.layer.resize(c->n_layers);
    for (int l = 0; l < c->n_layers; l++) {
        LayerPlan &y = p.layer[l];
        const int kb = c->kbits[l], vb = c->vbits[l];
        y.kcode = off; off = align_up(off + BH * p.NB * kvq::block_code_bytes(kb));
        y.kmeta = off; off = align_up(off + BH * p.NB * kvq::block_meta_bytes(kb, narrow));
        y.vcode = off; off = align_up(off + BH * p.NB * kvq::block_code_bytes(vb));
        y.vmeta = off; off = align_up(off + BH * p.NB * kvq::block_meta_bytes(vb, narrow));
        y.bexp = off; off = align_up(off + BH * p.NB * sizeof(uint32_t));
        y.kres = off; off = align_up(off + BH * p.RC * kvq::kD * 2);
        y.vres = off; off = align_up(off + BH * p.RC * kvq::kD * 2);
    }
    const size_t rows = (size_t)c->batch * c->n_q_heads;
    p.part_o = off; off = align_up(off + rows * kMaxSplits * kvq::kD * sizeof(float));
    p.part_ml = off; off = align_up(off + rows * kMaxSplits * 2 * sizeof(float));
    p.prefill_chunk = BH < (size_t)kPrefillChunk ? (int)BH : kPrefillChunk;
    p.prefill_scratch = off; off = align_up(off + (size_t)p.prefill_chunk * p.NB * kvq::prefill_unit_bytes());
    p.prefill_select = off; off = align_up(off + BH * kvq::prefill_select_bytes());       // (a pass may take all caches)
    p.total = off;
    return p;
}

}  // namespace

struct kvq_ctx {
    kvq_config cfg;
    std::vector<uint8_t> kbits, vbits;
    std::vector<int> tokens;        // T per layer
    Plan plan;
    uint8_t *ws;
    hipStream_t stream;
    int variant;                    // 0 auto, 1 vector ALU, 2 matrix core
    int splits;                     // 0 auto
    int prefill_low_parts;          // 0: chosen per cache, 1: every key channel keeps its low part
    hipEvent_t ev_begin, ev_end;    // recorded around the main decode kernel when both are set
};

namespace {

int decode_variant(const kvq_ctx *c) { return c->variant == 0 ? 2 : c->variant; }     // the matrix-core kernel is the default

int packed_tokens(const kvq_ctx *c, int T)
{
    const int over = T - c->cfg.residual;
    return over > 0 ? kvq::kG * (over / kvq::kG) : 0;
}

kvq::LayerView view(const kvq_ctx *c, int l)
{
    const LayerPlan &y = c->plan.layer[l];
    kvq::LayerView v;
    v.kcode = c->ws + y.kcode;
    v.kmeta = reinterpret_cast<float *>(c->ws + y.kmeta);
    v.vcode = c->ws + y.vcode;
    v.vmeta = reinterpret_cast<float *>(c->ws + y.vmeta);
    v.bexp = reinterpret_cast<uint32_t *>(c->ws + y.bexp);
    v.kres = reinterpret_cast<uint16_t *>(c->ws + y.kres);
    v.vres = reinterpret_cast<uint16_t *>(c->ws + y.vres);
    v.kbits = c->kbits[l];
    v.vbits = c->vbits[l];
    v.narrow = c->cfg.meta_dtype == KVQ_META_FP16 ? 1 : 0;
    v.kpt = c->cfg.key_mode == KVQ_KEYS_PER_TOKEN ? 1 : 0;
    return v;
}

float *ws_part_o(const kvq_ctx *c) { return reinterpret_cast<float *>(c->ws + c->plan.part_o); }
float *ws_part_ml(const kvq_ctx *c) { return reinterpret_cast<float *>(c->ws + c->plan.part_ml); }
size_t ws_part_records(const kvq_ctx *c) { return (size_t)c->cfg.batch * c->cfg.n_q_heads * kMaxSplits; }

int launch_failed(const char *what, hipError_t e)
{
    snprintf(g_last_error, sizeof g_last_error, "%s: %s", what, hipGetErrorString(e));
    return KVQ_ELAUNCH;
}

}  // namespace

extern "C" {

size_t kvq_workspace_bytes(const kvq_config *cfg)
{
    if (!config_ok(cfg)) return 0;
    return make_plan(cfg).total;
}

int kvq_configure(kvq_ctx **out, const kvq_config *cfg, void *workspace_device, size_t workspace_bytes,
                  void *hip_stream)
{
    if (!out) return KVQ_EINVAL;
    *out = nullptr;
    if (!config_ok(cfg)) return KVQ_EINVAL;
    Plan plan = make_plan(cfg);
    if (!workspace_device || (reinterpret_cast<uintptr_t>(workspace_device) % kAlign) || workspace_bytes < plan.total)
        return KVQ_EWORKSPACE;
    kvq_ctx *c = new (std::nothrow) kvq_ctx();
    if (!c) return KVQ_EINVAL;
    c->cfg = *cfg;
    c->kbits.assign(cfg->kbits, cfg->kbits + cfg->n_layers);
    c->vbits.assign(cfg->vbits, cfg->vbits + cfg->n_layers);
    c->cfg.kbits = c->kbits.data();
    c->cfg.vbits = c->vbits.data();
    c->tokens.assign(cfg->n_layers, 0);
    c->plan = plan;
    c->ws = static_cast<uint8_t *>(workspace_device);
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->variant = 0;
    c->splits = 0;
    c->prefill_low_parts = 0;
    c->ev_begin = c->ev_end = nullptr;
    *out = c;
    return KVQ_OK;
}

namespace {

// Append n_tokens to a layer: quantize the groups that leave the fp16 window, then (unless the caller's decode
// launch takes the single new token along) copy the tokens that stay in the window into the ring.
int append_tokens(kvq_ctx *c, int layer, const void *k_device, const void *v_device, int n_tokens, bool copy_window)
{
    const int t_old = c->tokens[layer];
    if ((int64_t)t_old + n_tokens > c->cfg.max_tokens) return KVQ_ECAPACITY;
    const int t_new = t_old + n_tokens;
    const int np_old = packed_tokens(c, t_old), np_new = packed_tokens(c, t_new);
    const int BH = c->cfg.batch * c->cfg.n_kv_heads;

    // 1. quantize the groups that leave the fp16 window: positions [np_old, np_new)
    if (np_new > np_old) {
        kvq::QuantArgs a;
        a.lv = view(c, layer);
        a.k_in = static_cast<const uint16_t *>(k_device);
        a.v_in = static_cast<const uint16_t *>(v_device);
        a.n_in = n_tokens;
        a.t_old = t_old;
        a.first_block = np_old / kvq::kG;
        a.n_blocks = (np_new - np_old) / kvq::kG;
        a.BH = BH;
        a.NB = c->plan.NB;
        a.RC = c->plan.RC;
        hipError_t e = kvq::launch_quantize(a, c->stream);
        if (e != hipSuccess) return launch_failed("quantize kernel", e);
    }
    // 2. new tokens that stay in the window go to the ring (after step 1 has read the old slots)
    const int pos0 = np_new > t_old ? np_new : t_old;
    if (copy_window && t_new > pos0) {
        kvq::ResidualCopyArgs a;
        a.lv = view(c, layer);
        a.k_in = static_cast<const uint16_t *>(k_device);
        a.v_in = static_cast<const uint16_t *>(v_device);
        a.n_in = n_tokens;
        a.t_old = t_old;
        a.pos0 = pos0;
        a.pos1 = t_new;
        a.BH = BH;
        a.RC = c->plan.RC;
        hipError_t e = kvq::launch_residual_copy(a, c->stream);
        if (e != hipSuccess) return launch_failed("window copy kernel", e);
    }
    c->tokens[layer] = t_new;
    return KVQ_OK;
}

// How a decode launch divides the tokens of a (batch, kv head) cache among its groups.
struct SplitPlan { int splits, units_per_split, split_rem; };

// BH caches, code width = key bits + value bits, n_blocks packed blocks and n_res fp16 window tokens per cache;
// forced: the caller's split count (0 = choose); variant: 1 vector-ALU kernel, 2 matrix-core kernel.
SplitPlan plan_splits(int BH, int width, int n_blocks, int n_res, int forced, int variant)
{
    int splits = forced;
    if (splits <= 0) {
        // 16 waves per compute unit (4 on every SIMD) over 256 compute units: 2048 two-wave groups of the
        // matrix-core kernel or 1024 four-wave groups of the vector kernel.  More splits only add per-group
        // set-up and merge work, so split no further and keep at least 4 (8) blocks per group.
        // The wider a layer's codes, the more bytes every group keeps in flight and the fewer groups serve it
        // best (measured at batch 8..64, 8K and 32K tokens: K8V8 4-7 % faster with 1024 groups than with 2048,
        // K8V4 and K4V8 5 %; K4V4 and narrower are fastest with 2048).  K8V2 and K2V8 are as fast with 1024 as with
        // 2048 and 2-6 % slower with 1536 (3 waves per SIMD: the key and value roles cannot be even on every SIMD).
        const int groups = variant != 2 ? 1024 : width <= 8 ? 2048 : 1024;
        const int min_units = variant == 2 ? 4 : 8;
        splits = (groups + BH - 1) / BH;
        const int cap = (n_blocks + min_units - 1) / min_units + (n_res > 0 ? 1 : 0);
        if (splits > cap) splits = cap;
    }
    if (splits > kMaxSplits) splits = kMaxSplits;
    if (splits < 1) splits = 1;
    // The fp16 window rides on the last split.  Its rows are fetched and used after the split's blocks, chunk by chunk
    // and the values after the keys: memory round trips in a row, which cost about as much as kWindowWeight packed
    // blocks per chunk.  The window counts as that many units behind the blocks, and the units are dealt out evenly
    // (the last split gets that many blocks fewer, none at all when its share is smaller than that).  Measured at
    // batch 16, 8192..8223 tokens: weights 6..10 for one chunk and 10..16 for two are alike; with 4 a two-chunk window
    // makes its split the straggler (36.5 us against 30.4).
    int window = kWindowWeight * ((n_res + 31) / 32);
    if (n_blocks == 0) splits = 1;
    const int most = n_blocks + (window ? 1 : 0);                // no more splits than blocks (+ one for the window)
    if (splits > most) splits = most;
    if (splits < 1) splits = 1;
    // (never more than a split's share of blocks: with many small splits the window's split simply takes no blocks)
    if (window > (n_blocks + splits - 1) / splits) window = (n_blocks + splits - 1) / splits;
    if (n_res > 0 && window < 1) window = 1;
    SplitPlan p;
    for (;;) {
        const int total = n_blocks + window;
        p.units_per_split = total / splits;
        p.split_rem = total % splits;
        if (splits <= 1) break;
        // No empty split: every split but the last must start inside the blocks (look at the one before the last), and
        // without a window so must the last.
        auto first_unit = [&](int sidx) { return sidx * p.units_per_split + (sidx > splits - p.split_rem ? sidx - (splits - p.split_rem) : 0); };
        if (first_unit(splits - 2) < n_blocks && (window || first_unit(splits - 1) < n_blocks)) break;
        splits--;
    }
    p.splits = splits;
    return p;
}

// Decode attention over the layer's tokens.  k_new / v_new: rows of a token that append_tokens() left out of the
// window ring (fused append), or NULL.
// part_o / part_ml: where the splits' partial results go, room for part_records (query row, split) records.
int decode_layer(kvq_ctx *c, int layer, const void *q_device, void *out_device, const void *k_new, const void *v_new,
                 float *part_o, float *part_ml, size_t part_records)
{
    const int T = c->tokens[layer];
    if (T < 1) return KVQ_ESTATE;
    const int np = packed_tokens(c, T);
    kvq::DecodeArgs a;
    a.lv = view(c, layer);
    a.q = static_cast<const uint16_t *>(q_device);
    a.out = static_cast<uint16_t *>(out_device);
    a.part_o = part_o;
    a.part_ml = part_ml;
    a.B = c->cfg.batch;
    a.Hq = c->cfg.n_q_heads;
    a.Hkv = c->cfg.n_kv_heads;
    a.n_blocks = np / kvq::kG;
    a.n_res = T - np;
    a.NB = c->plan.NB;
    a.RC = c->plan.RC;
    a.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)kvq::kD));
    a.k_new = static_cast<const uint16_t *>(k_new);
    a.v_new = static_cast<const uint16_t *>(v_new);
    a.new_pos = T - 1;
    const int variant = decode_variant(c);
    const SplitPlan sp = plan_splits(a.B * a.Hkv, a.lv.kbits + a.lv.vbits, a.n_blocks, a.n_res, c->splits, variant);
    const int splits = sp.splits;
    a.units_per_split = sp.units_per_split;
    a.split_rem = sp.split_rem;
    a.splits = splits;
    if ((size_t)a.B * a.Hq * (size_t)splits > part_records) {
        snprintf(g_last_error, sizeof g_last_error,
                 "decode needs %zu partial records (%d query rows x %d splits), the scratch holds %zu",
                 (size_t)a.B * a.Hq * (size_t)splits, a.B * a.Hq, splits, part_records);
        return KVQ_ESCRATCH;
    }
    const bool timed = c->ev_begin && c->ev_end;
    hipError_t e;
    if (variant == 2) {
        // the matrix-core kernel's dispatch stamps the two events itself (its own start and end, no marker in between)
        e = kvq::launch_decode_mfma(a, c->stream, timed ? c->ev_begin : nullptr, timed ? c->ev_end : nullptr);
    } else {
        if (timed && hipEventRecord(c->ev_begin, c->stream) != hipSuccess) return launch_failed("event record", hipGetLastError());
        e = kvq::launch_decode_valu(a, c->stream);
        if (e == hipSuccess && timed && hipEventRecord(c->ev_end, c->stream) != hipSuccess) return launch_failed("event record", hipGetLastError());
    }
    if (e != hipSuccess) return launch_failed("decode kernel", e);
    e = kvq::launch_combine(a, c->stream);
    if (e != hipSuccess) return launch_failed("combine kernel", e);
    return KVQ_OK;
}

}  // namespace

int kvq_quantize_append(kvq_ctx *c, int32_t layer, const void *k_device, const void *v_device, int32_t n_tokens)
{
    if (!c || layer < 0 || layer >= c->cfg.n_layers || !k_device || !v_device || n_tokens < 1) return KVQ_EINVAL;
    return append_tokens(c, layer, k_device, v_device, n_tokens, true);
}

int kvq_decode_attention(kvq_ctx *c, int32_t layer, const void *q_device, void *out_device)
{
    if (!c || layer < 0 || layer >= c->cfg.n_layers || !q_device || !out_device) return KVQ_EINVAL;
    return decode_layer(c, layer, q_device, out_device, nullptr, nullptr, ws_part_o(c), ws_part_ml(c), ws_part_records(c));
}

int kvq_decode_attention_noalloc(kvq_ctx *c, int32_t layer, const void *q_device, void *out_device)
{
    if (!c || layer < 0 || layer >= c->cfg.n_layers || !q_device || !out_device) return KVQ_EINVAL;
    // the device address of the built-in scratch array, looked up once per GPU with that GPU current
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return launch_failed("hipGetDevice", e);
    if (dev < 0 || dev >= kMaxDevices) {
        snprintf(g_last_error, sizeof g_last_error, "device ordinal %d beyond the %d this build keeps scratch addresses for", dev, kMaxDevices);
        return KVQ_ESCRATCH;
    }
    unsigned char *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        ptr = g_scratch_ptr[dev].load(std::memory_order_relaxed);
        if (!ptr) {
            e = hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch));
            if (e != hipSuccess || !ptr) return launch_failed("hipGetSymbolAddress(scratch)", e);
            g_scratch_ptr[dev].store(ptr, std::memory_order_release);
        }
    }
    // every record the merge reads is written by this call's decode kernel first: nothing has to start at zero
    return decode_layer(c, layer, q_device, out_device, nullptr, nullptr, reinterpret_cast<float *>(ptr),
                        reinterpret_cast<float *>(ptr + kStaticOutBytes), kStaticRecords);
}

int kvq_append_decode_attention(kvq_ctx *c, int32_t layer, const void *k_device, const void *v_device, const void *q_device,
                                void *out_device)
{
    if (!c || layer < 0 || layer >= c->cfg.n_layers || !k_device || !v_device || !q_device || !out_device) return KVQ_EINVAL;
    // the matrix-core kernel takes the new token along (if it stays in the fp16 window); otherwise copy it first
    const int t_old = c->tokens[layer], t_new = t_old + 1;
    const bool fused = decode_variant(c) == 2 && t_new <= c->cfg.max_tokens && t_new > packed_tokens(c, t_new);
    int rc = append_tokens(c, layer, k_device, v_device, 1, !fused);
    if (rc != KVQ_OK) return rc;
    rc = decode_layer(c, layer, q_device, out_device, fused ? k_device : nullptr, fused ? v_device : nullptr,
                      ws_part_o(c), ws_part_ml(c), ws_part_records(c));
    // A refused decode launch must not leave a token counted whose window rows the decode kernel was to store: the
    // layer goes back to its length before the call.  What was enqueued before the refusal (a flush of the oldest
    // window group, a window copy) only writes what a repeat of the call writes again, identically.
    if (rc != KVQ_OK) c->tokens[layer] = t_old;
    return rc;
}

int kvq_prefill_attention(kvq_ctx *c, int32_t layer, const void *q_device, int32_t n_q, void *out_device)
{
    if (!c || layer < 0 || layer >= c->cfg.n_layers || !q_device || !out_device) return KVQ_EINVAL;
    const int T = c->tokens[layer];
    if (T < 1) return KVQ_ESTATE;
    if (n_q < 1 || n_q > T) {
        snprintf(g_last_error, sizeof g_last_error, "kvq_prefill_attention: n_q = %d queries, the layer holds %d tokens", n_q, T);
        return KVQ_EINVAL;
    }
    const int np = packed_tokens(c, T);
    kvq::PrefillArgs a;
    a.lv = view(c, layer);
    a.q = static_cast<const uint16_t *>(q_device);
    a.out = static_cast<uint16_t *>(out_device);
    a.B = c->cfg.batch;
    a.Hq = c->cfg.n_q_heads;
    a.Hkv = c->cfg.n_kv_heads;
    a.n_blocks = np / kvq::kG;
    a.n_res = T - np;
    a.NB = c->plan.NB;
    a.RC = c->plan.RC;
    a.n_q = n_q;
    a.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)kvq::kD));
    a.scratch = c->ws + c->plan.prefill_scratch;
    a.select = nullptr;
    const bool timed = c->ev_begin && c->ev_end;
    const int BH = a.B * a.Hkv;
    // The caches are taken a chunk at a time: dequantize the chunk's packed units into the scratch area, attend.
    // The scratch area holds prefill_chunk caches of NB units; a shorter prompt leaves room for more caches per
    // pass (kept a multiple of the 8 XCDs, which the attention kernel's placement wants): fewer, larger launches.
    int chunk = c->plan.prefill_chunk;
    if (a.n_blocks > 0 && chunk < BH) {
        const long long fit = (long long)c->plan.prefill_chunk * c->plan.NB / a.n_blocks;
        if (fit >= BH) chunk = BH;
        else if (fit / 8 * 8 > chunk) chunk = (int)(fit / 8 * 8);
    } else if (a.n_blocks == 0) {
        chunk = BH;                                             // window only: nothing goes through the scratch area
    }
    // Keys quantized per channel: one kernel in front decides for every cache which channels keep the low parts of
    // their keys (one record per cache), unless the caller wants them kept for all.
    uint8_t *select = nullptr;
    bool begun = false;                                         // the first kernel of the call has taken ev_begin
    if (c->prefill_low_parts == 0 && a.lv.kbits < 16 && !a.lv.kpt && a.n_blocks > 0) {
        select = c->ws + c->plan.prefill_select;
        a.bh0 = 0;
        a.n_bh = BH;
        a.select = select;
        const hipError_t e = kvq::launch_prefill_select(a, c->stream, timed ? c->ev_begin : nullptr);
        if (e != hipSuccess) return launch_failed("prefill channel selection kernel", e);
        begun = true;
    }
    for (int bh0 = 0; bh0 < BH; bh0 += chunk) {
        a.bh0 = bh0;
        a.n_bh = BH - bh0 < chunk ? BH - bh0 : chunk;
        a.select = select ? select + (size_t)bh0 * kvq::prefill_select_bytes() : nullptr;
        const bool first = bh0 == 0 && !begun, last = bh0 + chunk >= BH;
        const hipError_t e = kvq::launch_prefill_attention(a, c->stream, timed && first ? c->ev_begin : nullptr,
                                                           timed && last ? c->ev_end : nullptr);
        if (e != hipSuccess) return launch_failed("prefill attention kernels", e);
    }
    return KVQ_OK;
}

int kvq_layer_tokens(const kvq_ctx *c, int32_t layer, int32_t *n_packed, int32_t *n_residual)
{
    if (!c || layer < 0 || layer >= c->cfg.n_layers || !n_packed || !n_residual) return KVQ_EINVAL;
    const int T = c->tokens[layer];
    *n_packed = packed_tokens(c, T);
    *n_residual = T - *n_packed;
    return KVQ_OK;
}

int kvq_reset(kvq_ctx *c, int32_t layer)
{
    if (!c || layer < -1 || layer >= c->cfg.n_layers) return KVQ_EINVAL;
    for (int l = 0; l < c->cfg.n_layers; l++)
        if (layer < 0 || l == layer) c->tokens[l] = 0;
    return KVQ_OK;
}

int kvq_debug_export(kvq_ctx *c, int32_t layer, void *k_codes, void *k_scale, void *k_zero, void *v_codes,
                     void *v_scale, void *v_zero, void *k_res, void *v_res)
{
    if (!c || layer < 0 || layer >= c->cfg.n_layers) return KVQ_EINVAL;
    const int T = c->tokens[layer];
    kvq::ExportArgs a;
    a.lv = view(c, layer);
    a.k_codes = static_cast<uint8_t *>(k_codes);
    a.v_codes = static_cast<uint8_t *>(v_codes);
    a.k_scale = static_cast<float *>(k_scale);
    a.k_zero = static_cast<float *>(k_zero);
    a.v_scale = static_cast<float *>(v_scale);
    a.v_zero = static_cast<float *>(v_zero);
    a.k_res = static_cast<uint16_t *>(k_res);
    a.v_res = static_cast<uint16_t *>(v_res);
    a.n_packed = packed_tokens(c, T);
    a.n_res = T - a.n_packed;
    a.BH = c->cfg.batch * c->cfg.n_kv_heads;
    a.NB = c->plan.NB;
    a.RC = c->plan.RC;
    if (T == 0) return KVQ_OK;
    hipError_t e = kvq::launch_export(a, c->stream);
    if (e != hipSuccess) return launch_failed("export kernel", e);
    return KVQ_OK;
}

int kvq_debug_split_plan(const kvq_config *cfg, int32_t layer, int32_t n_tokens, int32_t variant, int32_t forced_splits,
                         int32_t *splits, int32_t *units_per_split, int32_t *split_rem)
{
    if (!config_ok(cfg) || layer < 0 || layer >= cfg->n_layers || n_tokens < 1 || n_tokens > cfg->max_tokens || variant < 0 ||
        variant > 2 || forced_splits < 0 || forced_splits > kMaxSplits || !splits || !units_per_split || !split_rem)
        return KVQ_EINVAL;
    const int over = n_tokens - cfg->residual;
    const int np = over > 0 ? kvq::kG * (over / kvq::kG) : 0;
    const SplitPlan p = plan_splits(cfg->batch * cfg->n_kv_heads, cfg->kbits[layer] + cfg->vbits[layer], np / kvq::kG, n_tokens - np,
                                    forced_splits, variant == 0 ? 2 : variant);
    *splits = p.splits;
    *units_per_split = p.units_per_split;
    *split_rem = p.split_rem;
    return KVQ_OK;
}

int kvq_set_decode_options(kvq_ctx *c, int32_t variant, int32_t splits)
{
    if (!c || variant < 0 || variant > 2 || splits < 0 || splits > kMaxSplits) return KVQ_EINVAL;
    c->variant = variant;
    c->splits = splits;
    return KVQ_OK;
}

int kvq_set_prefill_options(kvq_ctx *c, int32_t low_parts)
{
    if (!c || low_parts < 0 || low_parts > 1) return KVQ_EINVAL;
    c->prefill_low_parts = low_parts;
    return KVQ_OK;
}

int kvq_set_kernel_events(kvq_ctx *c, void *begin_event, void *end_event)
{
    if (!c || (begin_event == nullptr) != (end_event == nullptr)) return KVQ_EINVAL;
    c->ev_begin = static_cast<hipEvent_t>(begin_event);
    c->ev_end = static_cast<hipEvent_t>(end_event);
    return KVQ_OK;
}

void kvq_destroy(kvq_ctx *c) { delete c; }

const char *kvq_strerror(int status)
{
    switch (status) {
    case KVQ_OK: return "ok";
    case KVQ_EINVAL: return "invalid argument (null pointer, layer index, bits, shape or group)";
    case KVQ_ECAPACITY: return "append exceeds max_tokens";
    case KVQ_ESTATE: return "layer holds no token";
    case KVQ_EWORKSPACE: return "workspace missing, misaligned or too small";
    case KVQ_ELAUNCH: return "HIP launch failed";
    case KVQ_ESCRATCH: return "the call needs more scratch than the library's built-in array holds";
    default: return "unknown status";
    }
}

const char *kvq_last_error(void) { return g_last_error; }

}  // extern "C"
