// C-ABI entry points of libvispec_verify: host-side argument checks, launch planning and
// kernel enqueues. Nothing here allocates device memory or synchronises.
#include <math.h>
#include <string.h>

#include <atomic>

#include "vs_internal.h"

namespace {

using namespace vs;

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
inline bool is_pow2(int32_t x) { return x > 0 && (x & (x - 1)) == 0; }
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

} // namespace

namespace vs {
// Is the current device one this library's kernels were written for? Asked once per device
// and remembered; called after the argument checks and before the first enqueue.
int32_t check_device() {
    constexpr int kMaxDevices = 64;
    static std::atomic<int> known[kMaxDevices]; // 0 = not asked yet, 1 = gfx950, -1 = something else
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) {
        (void)hipGetLastError();
        return VS_ERR_NO_DEVICE;
    }
    if (dev < kMaxDevices) {
        const int k = known[dev].load(std::memory_order_relaxed);
        if (k != 0) return k > 0 ? VS_OK : VS_ERR_NO_DEVICE;
    }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        (void)hipGetLastError();
        return VS_ERR_NO_DEVICE;
    }
    const bool ok = strncmp(prop.gcnArchName, "gfx950", 6) == 0;
    if (dev < kMaxDevices) known[dev].store(ok ? 1 : -1, std::memory_order_relaxed);
    return ok ? VS_OK : VS_ERR_NO_DEVICE;
}
} // namespace vs

namespace {

struct Plan {
    int32_t impl, rpw, waves, row_groups, rows, rows_pad, num_splits, keys_per_split, total_wgs, schedule;
    int32_t bal_chunks; // balanced schedule: shares per (KV head, row group); num_splits = slots per KV head
    int32_t res_rb; // resident schedule: row blocks per workgroup (4, 2 or 1)
};

// Shape / dtype / layout checks that need no device. Returns VS_OK or a vs_error.
int32_t check_desc(const vs_attn_desc* d, int tree = 1) {
    if (!d) return VS_ERR_NULL;
    if (d->B < 1 || d->T < 1 || d->T > VS_MAX_TREE || d->Hq < 1 || d->Hkv < 1 || d->Hq % d->Hkv != 0)
        return VS_ERR_SHAPE;
    if (d->d != 64 && d->d != 128) return VS_ERR_SHAPE;
    if ((int64_t)d->B * d->Hkv > kMaxGridY) return VS_ERR_SHAPE; // one grid row per (sequence, KV head) in the combine
    if (d->max_prefix_len < 0) return VS_ERR_SHAPE;
    if (!(d->softmax_scale > 0.f) || !isfinite(d->softmax_scale)) return VS_ERR_SHAPE;
    if (d->dtype != VS_BF16 && d->dtype != VS_F32) return VS_ERR_DTYPE;
    if (d->impl != VS_IMPL_AUTO && d->impl != VS_IMPL_GENERIC && d->impl != VS_IMPL_MFMA) return VS_ERR_SHAPE;
    if (d->impl == VS_IMPL_MFMA && d->dtype != VS_BF16) return VS_ERR_DTYPE;
    if (d->num_splits < 0 || d->rows_per_wave < 0 || d->rows_per_wave > 2) return VS_ERR_SHAPE;
    if (d->waves_per_group != 0 && d->waves_per_group != 1 && d->waves_per_group != 2 && d->waves_per_group != 4 &&
        d->waves_per_group != 8)
        return VS_ERR_SHAPE;
    if (d->schedule != VS_SCHED_AUTO && d->schedule != VS_SCHED_LOOP && d->schedule != VS_SCHED_PIPELINED &&
        d->schedule != VS_SCHED_RESIDENT && d->schedule != VS_SCHED_BALANCED)
        return VS_ERR_SHAPE;
    if (d->schedule == VS_SCHED_RESIDENT && (d->rows_per_wave == 2 || (d->waves_per_group != 0 && d->waves_per_group != 8)))
        return VS_ERR_SHAPE; // eight waves, one row block each
    if (d->schedule == VS_SCHED_BALANCED) {
        // a lane per sequence and per share; num_splits, when given, is the number of shares
        if (d->B > kBalMaxSeqs || d->num_splits > kBalMaxChunks) return VS_ERR_SHAPE;
        if (d->impl == VS_IMPL_GENERIC || d->dtype != VS_BF16) return VS_ERR_SHAPE;
    }
    if (d->schedule == VS_SCHED_PIPELINED || d->schedule == VS_SCHED_BALANCED) {
        // the pipelined kernel exists for one row block per wave and four or eight waves
        if (d->rows_per_wave == 2) return VS_ERR_SHAPE;
        if (d->waves_per_group != 0 && d->waves_per_group != 4 && d->waves_per_group != 8) return VS_ERR_SHAPE;
    }
    if (d->stride_head < 0 || d->stride_tok < d->d) return VS_ERR_LAYOUT;
    const int64_t need = (int64_t)d->max_prefix_len + (tree ? d->T : 0);
    if (!tree && d->max_prefix_len < 1) return VS_ERR_SHAPE;
    if (d->paged) {
        if (!is_pow2(d->block_size) || d->block_size < 16) return VS_ERR_LAYOUT;
        if (d->max_blocks < 1 || d->num_blocks < 1 || d->stride_block < 0) return VS_ERR_LAYOUT;
        if (!d->block_table) return VS_ERR_NULL;
        if (need > (int64_t)d->max_blocks * d->block_size) return VS_ERR_LAYOUT;
    } else {
        if (d->stride_seq < 0 || d->capacity < 1) return VS_ERR_LAYOUT;
        if (need > d->capacity) return VS_ERR_LAYOUT;
    }
    const bool mfma = d->impl == VS_IMPL_MFMA || (d->impl == VS_IMPL_AUTO && d->dtype == VS_BF16);
    if (mfma) {
        // token offsets inside one (sequence, KV head) slice are kept in 32 bits
        const int64_t span = d->paged ? (int64_t)d->block_size * d->stride_tok : need * d->stride_tok;
        if (span >= ((int64_t)1 << 30)) return VS_ERR_LAYOUT;
        // 16-byte vector loads of 8 bf16
        if (d->stride_head % 8 || d->stride_tok % 8 || (d->paged ? d->stride_block % 8 : d->stride_seq % 8))
            return VS_ERR_LAYOUT;
    }
    return VS_OK;
}

Plan make_plan(const vs_attn_desc* d, int tree = 1) {
    Plan pl{};
    const int group = d->Hq / d->Hkv;
    pl.rows = d->T * group;
    pl.rows_pad = (pl.rows + kRowBlock - 1) / kRowBlock * kRowBlock;
    pl.impl = d->impl == VS_IMPL_AUTO ? (d->dtype == VS_BF16 ? VS_IMPL_MFMA : VS_IMPL_GENERIC) : d->impl;
    if (pl.impl == VS_IMPL_GENERIC) {
        pl.rpw = 0;
        pl.waves = 1;
        pl.row_groups = 1;
        pl.num_splits = 1;
        pl.keys_per_split = 0;
        pl.total_wgs = d->B * d->T * d->Hq;
        return pl;
    }
    const int nrb = pl.rows_pad / kRowBlock;
    const int tiles = ((int64_t)d->max_prefix_len + (tree ? d->T : 0) + kIterKeys - 1) / kIterKeys;
    const int units0 = d->B * d->Hkv;
    // Launch shape, from measurements on MI355X (C2..C5-shaped inputs):
    //  * few units (one layer of one sequence): latency-bound; straight-loop kernel, one
    //    row block per wave, at most four waves, more row groups and about 1.5 workgroups
    //    per CU;
    //  * many units: the software-pipelined kernel with one row block per wave, the rows
    //    split over row groups of eight (or four) waves, and key splits only when units x
    //    row groups leave CUs empty. No partial results when that alone fills the machine.
    //  * a caller who fixes rows_per_wave = 2 or a wave count the pipelined kernel does not
    //    have gets the straight loop: one row block per wave unless told otherwise, up to four
    //    waves for small launches and eight for large ones.
    const bool big = units0 >= kManyUnits;
    int rpw = d->rows_per_wave, waves = d->waves_per_group, splits = d->num_splits;
    const bool pipe_ok = (rpw == 0 || rpw == 1) && (waves == 0 || waves == 4 || waves == 8);
    const bool many = units0 >= 12; // enough (sequence, KV head) units for the pipelined kernel, see below
    // few units, several row blocks, a short sequence (at most 2048 keys) and no caller's
    // choice that it cannot honour: the LDS-resident kernel, whose second split of the keys
    // among the waves shortens each workgroup's loop - as long as all its workgroups (up to 96 KB
    // of LDS each: one per CU) run at once. Splits of two 64-key tiles when that fits, else
    // three. Measured on C3-sized layers replayed from a HIP graph over 400 MB of K/V (every
    // layer cold in the caches), per layer: 14 splits of 128 keys 15.8 us, 10 splits of 192 keys
    // 16.7 us; the streaming loop with the same splits 15.7 / 16.9 us. With two sequences (more
    // workgroups than CUs) it loses to the loop, and for 5000+ keys its 192-key limit forces too
    // many partial results.
    const int res_rg = (nrb + 3) / 4;
    const int res_tps = (int64_t)units0 * res_rg * ((tiles + 1) / 2) <= kNumCUs ? 2 : 3; // 64-key tiles per split
    const int res_splits = splits > 0 ? splits : (tiles + res_tps - 1) / res_tps;
    const bool resident_ok = !many && nrb >= 3 && tiles <= 32 && (rpw == 0 || rpw == 1) && (waves == 0 || waves == 8) &&
                             (splits <= 0 || (tiles + splits - 1) / splits <= kResidentMaxKeys / kIterKeys) &&
                             (int64_t)units0 * res_rg * res_splits <= kNumCUs;
    // The pipelined kernel takes over from twelve units on (three C3 sequences, or one MHA
    // layer): A/B per call, loop against pipelined, 3 sequences 26.3 / 24.9 us, 4: 28.6 / 26.9,
    // 6: 34.0 / 29.7, 8: 39.9 / 31.4, 11: 50.9 / 39.9, one C2 (MHA) layer 25.4 / 23.3; below
    // that the loop wins (one C3 sequence 19.1 / 22.5, two 21.7 / 23.3).
    // Balanced shares instead of equal splits per sequence: for batches whose sequences may differ in
    // length (the host only knows the longest allowed one). As many workgroups as the CUs hold at once
    // (one of eight waves, two of four). Taken when the launch would need key splits to fill those
    // places anyway, or when whole sequences would make more than one round and less than two - shares
    // then replace a second, partly filled round of workgroups of unequal length - and a share would
    // be 32 steps of 64 keys if every sequence had the longest allowed length (reading the lengths and
    // cutting the shares costs each kernel a dependent load and a few microseconds).
    // Paged batches, one layer, planner's other choice / balanced shares, lengths drawn from 1024 .. 8192
    // unless stated. Qwen-7B heads (28 / 4), 16 sequences: 138 / 118, 135 / 107, 138 / 106, 127 / 96 us; all
    // 4600 keys: 93 / 98; all 8000: 150 / 156; 256 .. 2048 keys: 50 / 57; 32 sequences: 242 / 192;
    // 40: 279 / 226, all 3000 keys 202 / 162; 64: 418 / 340, all 3000 keys 227 / 237. LLaVA-7B heads (32 / 32),
    // 4 sequences: 120 / 77; 8: 237 / 168; 12: 262 / 201; 24: 422 / 361; 32: 518 / 487, and 32 folded layers
    // of 3136 keys 308 / 334.
    // A launch that is one full round of whole sequences is left alone: unequal lengths would gain
    // there too, equal ones lose the second kernel and the wait for the lengths (7 us of 60), and the
    // host cannot tell which it has - such callers ask for VS_SCHED_BALANCED themselves. Two rounds or
    // more are left alone as well: the gain shrinks with every round and equal lengths lose 4 - 8 %.
    const int bal_waves = waves ? waves : (nrb > 4 ? 8 : 4);
    const int bal_rg = (nrb + bal_waves - 1) / bal_waves;
    const int bal_places = kNumCUs * (bal_waves == 8 ? 1 : 2);
    const int bal_w_auto = bal_places / (d->Hkv * bal_rg) > kBalMaxChunks ? kBalMaxChunks : bal_places / (d->Hkv * bal_rg);
    const int bal_wgs = units0 * bal_rg;
    const bool balanced_ok = many && pipe_ok && splits <= 0 && d->B >= 2 && d->B <= kBalMaxSeqs &&
                             (bal_wgs * 32 < bal_places * 25 || (bal_wgs > bal_places && bal_wgs < 2 * bal_places)) &&
                             bal_w_auto >= 2 && (int64_t)d->B * tiles >= 32 * (int64_t)bal_w_auto;
    pl.schedule = d->schedule != VS_SCHED_AUTO ? d->schedule
                  : balanced_ok                ? VS_SCHED_BALANCED
                  : many && pipe_ok            ? VS_SCHED_PIPELINED
                  : resident_ok                ? VS_SCHED_RESIDENT
                                               : VS_SCHED_LOOP;
    if (pl.schedule == VS_SCHED_BALANCED) {
        pl.rpw = 1;
        pl.waves = bal_waves;
        pl.row_groups = bal_rg;
        pl.bal_chunks = splits > 0 ? splits : (bal_w_auto < 1 ? 1 : bal_w_auto);
        pl.num_splits = pl.bal_chunks + d->B; // partial-result slots per KV head
        pl.keys_per_split = 0;                // shares are measured at run time
        pl.total_wgs = pl.bal_chunks * d->Hkv * pl.row_groups;
        return pl;
    }
    if (pl.schedule == VS_SCHED_RESIDENT) {
        // eight waves = res_rb row blocks x 8 / res_rb key parts; a split holds at most
        // kResidentMaxKeys keys (three 64-key tiles)
        pl.rpw = 1;
        pl.waves = 8;
        pl.res_rb = nrb >= 3 ? 4 : nrb;
        pl.row_groups = (nrb + pl.res_rb - 1) / pl.res_rb;
        const int max_tiles = kResidentMaxKeys / kIterKeys;
        if (splits <= 0) splits = res_splits;
        int tps = (tiles + splits - 1) / splits;
        if (tps > max_tiles) tps = max_tiles;
        if (tps < 1) tps = 1;
        pl.keys_per_split = tps * kIterKeys;
        pl.num_splits = (tiles + tps - 1) / tps;
        pl.total_wgs = units0 * pl.row_groups * pl.num_splits;
        return pl;
    }
    if (pl.schedule == VS_SCHED_PIPELINED) {
        rpw = 1;
        if (!waves) waves = nrb > 4 ? 8 : 4;
        if (splits <= 0) {
            const int wgs = units0 * ((nrb + waves - 1) / waves);
            splits = wgs >= 200 ? 1 : kNumCUs / wgs;
            const int max_splits = (tiles + 3) / 4; // at least four iterations per split
            if (splits > max_splits) splits = max_splits;
        }
    } else {
        if (!rpw) rpw = 1;
        if (!waves) {
            const int need1 = (nrb + rpw - 1) / rpw;
            const int cap = (big && nrb > 4) ? kMaxWaves : 4;
            waves = 1;
            while (waves < need1 && waves < cap) waves *= 2;
        }
    }
    pl.rpw = rpw;
    pl.waves = waves;
    const int need = (nrb + pl.rpw - 1) / pl.rpw;
    pl.row_groups = (need + pl.waves - 1) / pl.waves;
    const int units = units0 * pl.row_groups;
    if (splits <= 0) {
        // large: fill the CUs once. Small launches are latency-bound: the write-back of the
        // partial results at the end of the kernel (about 0.2 us per split for a C3-sized
        // launch) and the combine grow with the split count, the loop (about 2 us per 64 keys
        // with one wave per SIMD) with the keys per split; measured optima were 3 iterations
        // of 64 keys per split for short sequences and 8 for long ones, with at most one
        // workgroup per CU (two C3 sequences: 7 splits = 224 workgroups 21.7 us, 10 splits = 320
        // workgroups 25.1 us).
        if (big) {
            splits = kNumCUs / units;
        } else {
            const int iters = tiles <= 32 ? 3 : (tiles <= 64 ? 5 : 8);
            splits = (tiles + iters - 1) / iters;
            const int cap = kNumCUs / units; // one workgroup per CU: a second one on some CUs makes those the tail
            if (splits > cap) splits = cap;
        }
        const int max_splits = (tiles + 1) / 2;
        if (splits > max_splits) splits = max_splits;
    }
    if (splits < 1) splits = 1;
    if (splits > tiles) splits = tiles;
    if (splits > 64) splits = 64; // more splits than this only add partial-result traffic
    const int tiles_per_split = (tiles + splits - 1) / splits;
    pl.keys_per_split = tiles_per_split * kIterKeys;
    pl.num_splits = (tiles + tiles_per_split - 1) / tiles_per_split;
    pl.total_wgs = units * pl.num_splits;
    return pl;
}

// rows of partial results: every (sequence, KV head) has num_splits slots; the balanced schedule has
// num_splits slots per KV head for the whole batch
size_t partial_rows(const vs_attn_desc* d, const Plan& pl) {
    return (size_t)(pl.bal_chunks > 0 ? 1 : d->B) * d->Hkv * pl.num_splits * pl.rows_pad;
}

size_t workspace_bytes(const vs_attn_desc* d, const Plan& pl) {
    if (pl.impl != VS_IMPL_MFMA || pl.num_splits <= 1) return 0;
    const size_t prow = partial_rows(d, pl);
    return align_up(prow * d->d * sizeof(uint16_t)) + align_up(prow * 2 * sizeof(float)) +
           (pl.bal_chunks > 0 ? align_up(kBalMaxChunks * sizeof(int32_t)) : 0);
}

constexpr int kArgmaxChunk = kAcceptChunk;

int32_t accept_chunks(int32_t V) { return (V + kArgmaxChunk - 1) / kArgmaxChunk; }

} // namespace

extern "C" {

int32_t vs_version(void) { return VS_VERSION; }

const char* vs_strerror(int32_t err) {
    switch (err) {
    case VS_OK: return "ok";
    case VS_ERR_NULL: return "a required pointer is NULL";
    case VS_ERR_SHAPE: return "unsupported or inconsistent shape";
    case VS_ERR_DTYPE: return "unsupported dtype";
    case VS_ERR_WORKSPACE: return "workspace missing or too small";
    case VS_ERR_HIP: return "HIP runtime error at launch";
    case VS_ERR_LAYOUT: return "unsupported strides, alignment or paging parameters";
    case VS_ERR_NO_DEVICE: return "no usable gfx950 device";
    default: return "unknown error";
    }
}

const char* vs_status_string(int32_t code) {
    switch (code) {
    case VS_STATUS_OK: return "ok";
    case VS_STATUS_BAD_ROOT: return "parent[0] is not -1";
    case VS_STATUS_BAD_PARENT: return "a parent index is outside [0, i)";
    case VS_STATUS_BAD_PREFIX: return "prefix_len outside the cache or the host bound";
    case VS_STATUS_BAD_BLOCK: return "a block-table entry is outside the pool";
    case VS_STATUS_BAD_PATH: return "accepted path is not the root followed by increasing node ids";
    case VS_STATUS_BAD_CANDIDATE: return "a candidate's parent is not an earlier candidate, or a child outscores its parent";
    default: return "unknown status";
    }
}

int32_t vs_tree_validate_host(const int32_t* parent, int32_t T) {
    if (!parent) return VS_ERR_NULL;
    if (T < 1 || T > VS_MAX_TREE) return VS_ERR_SHAPE;
    return validate_tree_host(parent, T);
}

int32_t vs_tree_mask_build(const int32_t* parent, int32_t B, int32_t T, uint64_t* mask, int32_t* depth,
                           int32_t* status, void* stream) {
    if (!parent || !mask || !depth) return VS_ERR_NULL;
    if (B < 1 || T < 1 || T > VS_MAX_TREE) return VS_ERR_SHAPE;
    if (const int32_t dc = check_device()) return dc;
    return launch_tree_mask(parent, B, T, mask, depth, status, (hipStream_t)stream) == hipSuccess ? VS_OK
                                                                                                    : VS_ERR_HIP;
}

int32_t vs_attention_plan(const vs_attn_desc* desc, vs_attn_plan* plan) {
    if (!plan) return VS_ERR_NULL;
    const int32_t rc = check_desc(desc);
    if (rc != VS_OK) return rc;
    const Plan pl = make_plan(desc);
    plan->impl = pl.impl;
    plan->num_splits = pl.bal_chunks > 0 ? pl.bal_chunks : pl.num_splits;
    plan->keys_per_split = pl.keys_per_split;
    plan->row_groups = pl.row_groups;
    plan->waves_per_group = pl.waves;
    plan->rows_per_wave = pl.rpw;
    plan->workgroups = pl.total_wgs;
    plan->combine = (pl.impl == VS_IMPL_MFMA && pl.num_splits > 1) ? 1 : 0;
    plan->schedule = pl.schedule;
    return VS_OK;
}

size_t vs_attention_workspace_bytes(const vs_attn_desc* desc) {
    if (check_desc(desc) != VS_OK) return 0;
    return workspace_bytes(desc, make_plan(desc));
}

namespace {
// Shared by the two attention entry points. tree = 1: the T queries are tree nodes whose own
// K/V sit behind the prefix; tree = 0: T learnable queries over the prefix alone.
int32_t enqueue_attention(const vs_attn_desc* desc, int tree, const void* q, const void* k_cache, const void* v_cache,
                          const int32_t* prefix_len, const int32_t* tree_parent, const uint64_t* tree_mask, void* out,
                          int32_t* status, void* workspace, size_t workspace_bytes_given, void* stream) {
    const int32_t rc = check_desc(desc, tree);
    if (rc != VS_OK) return rc;
    const Plan pl = make_plan(desc, tree);
    if (pl.impl == VS_IMPL_MFMA && !(aligned16(q) && aligned16(k_cache) && aligned16(v_cache) && aligned16(out)))
        return VS_ERR_LAYOUT;
    const size_t need = workspace_bytes(desc, pl);
    if (need > 0 && (!workspace || workspace_bytes_given < need || ((uintptr_t)workspace & (kAlign - 1))))
        return VS_ERR_WORKSPACE;
    if (const int32_t dc = check_device()) return dc;

    AttnParams p{};
    p.q = q;
    p.k = k_cache;
    p.v = v_cache;
    p.out = out;
    p.prefix_len = prefix_len;
    p.parent = tree_parent;
    p.tree_mask = tree_mask;
    p.block_table = desc->paged ? desc->block_table : nullptr;
    p.status = status;
    p.B = desc->B;
    p.T = desc->T;
    p.tree_keys = tree ? desc->T : 0;
    p.Hq = desc->Hq;
    p.Hkv = desc->Hkv;
    p.d = desc->d;
    p.group = desc->Hq / desc->Hkv;
    p.rows = pl.rows;
    p.rows_pad = pl.rows_pad;
    p.max_prefix_len = desc->max_prefix_len;
    p.paged = desc->paged ? 1 : 0;
    p.block_size = desc->paged ? desc->block_size : 1;
    p.block_shift = 0;
    while ((1 << p.block_shift) < p.block_size) ++p.block_shift;
    p.max_blocks = desc->max_blocks;
    p.num_blocks = desc->num_blocks;
    p.capacity = desc->capacity;
    p.stride_seq = desc->stride_seq;
    p.stride_block = desc->stride_block;
    p.stride_head = desc->stride_head;
    p.stride_tok = desc->stride_tok;
    p.scale = desc->softmax_scale;
    p.scale_log2 = desc->softmax_scale * 1.4426950408889634f;
    p.num_splits = pl.num_splits;
    p.keys_per_split = pl.keys_per_split;
    p.row_groups = pl.row_groups;
    p.rows_per_group = (pl.schedule == VS_SCHED_RESIDENT ? pl.res_rb : pl.waves * pl.rpw) * kRowBlock;
    p.total_wgs = pl.total_wgs;
    p.bal_chunks = pl.bal_chunks;
    if (need > 0) {
        const size_t prow = partial_rows(desc, pl);
        p.part_o = (uint16_t*)workspace;
        p.part_ml = (float*)((char*)workspace + align_up(prow * desc->d * sizeof(uint16_t)));
        if (pl.bal_chunks > 0) p.bal_table = (int32_t*)((char*)p.part_ml + align_up(prow * 2 * sizeof(float)));
    }
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    if (pl.impl == VS_IMPL_GENERIC) {
        e = launch_attention_generic(p, desc->dtype, s);
    } else {
        e = (pl.schedule == VS_SCHED_PIPELINED || pl.schedule == VS_SCHED_BALANCED) ? launch_attention_mfma_pipe(p, pl.rpw, pl.waves, s)
            : pl.schedule == VS_SCHED_RESIDENT ? launch_attention_mfma_resident(p, pl.res_rb, s)
                                               : launch_attention_mfma(p, pl.rpw, pl.waves, s);
        if (e == hipSuccess && pl.num_splits > 1) e = launch_attention_combine(p, desc->dtype, s);
    }
    return e == hipSuccess ? VS_OK : VS_ERR_HIP;
}
} // namespace

int32_t vs_tree_verify_attention(const vs_attn_desc* desc, const void* q, const void* k_cache,
                                 const void* v_cache, const int32_t* prefix_len, const int32_t* tree_parent,
                                 const uint64_t* tree_mask, void* out, int32_t* status, void* workspace,
                                 size_t workspace_bytes_given, void* stream) {
    if (!desc || !q || !k_cache || !v_cache || !prefix_len || !tree_parent || !out) return VS_ERR_NULL;
    return enqueue_attention(desc, 1, q, k_cache, v_cache, prefix_len, tree_parent, tree_mask, out, status, workspace,
                             workspace_bytes_given, stream);
}

size_t vs_compress_attention_workspace_bytes(const vs_attn_desc* desc) {
    if (check_desc(desc, 0) != VS_OK) return 0;
    return workspace_bytes(desc, make_plan(desc, 0));
}

int32_t vs_compress_attention(const vs_attn_desc* desc, const void* q, const void* k, const void* v,
                              const int32_t* kv_len, void* out, int32_t* status, void* workspace,
                              size_t workspace_bytes_given, void* stream) {
    if (!desc || !q || !k || !v || !kv_len || !out) return VS_ERR_NULL;
    return enqueue_attention(desc, 0, q, k, v, kv_len, nullptr, nullptr, out, status, workspace, workspace_bytes_given,
                             stream);
}

size_t vs_accept_workspace_bytes(int32_t B, int32_t T, int32_t V) {
    if (B < 1 || T < 1 || T > VS_MAX_TREE || V < 1) return 0;
    const size_t n = (size_t)B * T * accept_chunks(V);
    return align_up(n * sizeof(float)) + align_up(n * sizeof(int32_t));
}

int32_t vs_tree_accept(const float* logits, int64_t ld_logits, int32_t V, const int32_t* draft_tokens,
                       const int32_t* parent, int32_t B, int32_t T, int32_t* accepted_len, int32_t* path,
                       int32_t* bonus_token, int32_t* row_argmax, int32_t* status, void* workspace,
                       size_t workspace_bytes_given, void* stream) {
    if (!logits || !draft_tokens || !parent || !accepted_len || !path || !bonus_token) return VS_ERR_NULL;
    if (B < 1 || T < 1 || T > VS_MAX_TREE || V < 1 || ld_logits < V) return VS_ERR_SHAPE;
    if ((int64_t)B * T * accept_chunks(V) > kMaxGridX) return VS_ERR_SHAPE; // one workgroup per (row, chunk)
    const size_t need = vs_accept_workspace_bytes(B, T, V);
    if (!workspace || workspace_bytes_given < need || ((uintptr_t)workspace & (kAlign - 1))) return VS_ERR_WORKSPACE;
    if (const int32_t dc = check_device()) return dc;
    AcceptParams p{};
    p.logits = logits;
    p.ld = ld_logits;
    p.V = V;
    p.draft = draft_tokens;
    p.parent = parent;
    p.B = B;
    p.T = T;
    p.accepted_len = accepted_len;
    p.path = path;
    p.bonus = bonus_token;
    p.row_argmax = row_argmax;
    p.status = status;
    p.chunks = accept_chunks(V);
    p.chunk_elems = kArgmaxChunk;
    p.vec_ok = (aligned16(logits) && ld_logits % 4 == 0) ? 1 : 0;
    const size_t n = (size_t)B * T * p.chunks;
    p.part_val = (float*)workspace;
    p.part_idx = (int32_t*)((char*)workspace + align_up(n * sizeof(float)));
    return launch_accept(p, (hipStream_t)stream) == hipSuccess ? VS_OK : VS_ERR_HIP;
}

size_t vs_accept_sample_workspace_bytes(int32_t B, int32_t T, int32_t V) {
    if (B < 1 || T < 1 || T > VS_MAX_TREE || V < 1 || accept_chunks(V) > kMaxSampleChunks) return 0;
    const size_t n = (size_t)B * T * accept_chunks(V);
    return 2 * align_up(n * sizeof(float));
}

int32_t vs_tree_accept_sample(const float* logits, int64_t ld_logits, int32_t V, float temperature,
                              const int32_t* draft_tokens, const int32_t* parent, const float* u_accept,
                              const float* u_bonus, int32_t B, int32_t T, int32_t* accepted_len, int32_t* path,
                              int32_t* bonus_token, int32_t* status, void* workspace, size_t workspace_bytes_given,
                              void* stream) {
    if (!logits || !draft_tokens || !parent || !u_accept || !u_bonus || !accepted_len || !path || !bonus_token)
        return VS_ERR_NULL;
    if (B < 1 || T < 1 || T > VS_MAX_TREE || V < 1 || ld_logits < V) return VS_ERR_SHAPE;
    if (accept_chunks(V) > kMaxSampleChunks || (int64_t)B * T * accept_chunks(V) > kMaxGridX) return VS_ERR_SHAPE;
    if (!(temperature > 0.f) || !(temperature < INFINITY)) return VS_ERR_SHAPE;
    const size_t need = vs_accept_sample_workspace_bytes(B, T, V);
    if (!workspace || workspace_bytes_given < need || ((uintptr_t)workspace & (kAlign - 1))) return VS_ERR_WORKSPACE;
    if (const int32_t dc = check_device()) return dc;
    SampleParams p{};
    p.logits = logits;
    p.ld = ld_logits;
    p.V = V;
    p.draft = draft_tokens;
    p.parent = parent;
    p.u_accept = u_accept;
    p.u_bonus = u_bonus;
    p.B = B;
    p.T = T;
    p.accepted_len = accepted_len;
    p.path = path;
    p.bonus = bonus_token;
    p.status = status;
    p.k_log2 = 1.4426950408889634f / temperature;
    p.chunks = accept_chunks(V);
    p.chunk_elems = kArgmaxChunk;
    p.vec_ok = (aligned16(logits) && ld_logits % 4 == 0) ? 1 : 0;
    const size_t n = (size_t)B * T * p.chunks;
    p.part_m = (float*)workspace;
    p.part_s = (float*)((char*)workspace + align_up(n * sizeof(float)));
    return launch_accept_sample(p, (hipStream_t)stream) == hipSuccess ? VS_OK : VS_ERR_HIP;
}

size_t vs_draft_expand_workspace_bytes(int32_t B, int32_t F, int32_t V, int32_t K) {
    if (B < 1 || F < 1 || F > VS_MAX_TREE || K < 1 || K > kMaxDraftK || F * K > kMaxDraftCand || V < K) return 0;
    const size_t n = (size_t)B * F * accept_chunks(V);
    return 2 * align_up(n * sizeof(float)) + 2 * align_up(n * K * sizeof(float));
}

int32_t vs_draft_expand(const float* logits, int64_t ld_logits, int32_t V, const float* cum_in,
                        const int32_t* frontier_cand, int32_t B, int32_t F, int32_t K, int32_t cand_base,
                        int32_t cand_capacity, int32_t* cand_token, float* cand_score, int32_t* cand_parent,
                        int32_t* next_frontier_cand, float* next_cum, void* workspace, size_t workspace_bytes_given,
                        void* stream) {
    if (!logits || !cand_token || !cand_score || !cand_parent || !next_frontier_cand || !next_cum) return VS_ERR_NULL;
    if (B < 1 || F < 1 || F > VS_MAX_TREE || K < 1 || K > kMaxDraftK || F * K > kMaxDraftCand) return VS_ERR_SHAPE;
    if (V < K || ld_logits < V || (int64_t)B * F * accept_chunks(V) > kMaxGridX) return VS_ERR_SHAPE;
    if (cand_base < 0 || cand_capacity < 1 || (int64_t)cand_base + (int64_t)F * K > cand_capacity) return VS_ERR_SHAPE;
    const size_t need = vs_draft_expand_workspace_bytes(B, F, V, K);
    if (!workspace || workspace_bytes_given < need || ((uintptr_t)workspace & (kAlign - 1))) return VS_ERR_WORKSPACE;
    if (const int32_t dc = check_device()) return dc;
    DraftExpandParams p{};
    p.logits = logits;
    p.ld = ld_logits;
    p.V = V;
    p.cum_in = cum_in;
    p.frontier_cand = frontier_cand;
    p.B = B;
    p.F = F;
    p.K = K;
    p.cand_base = cand_base;
    p.cand_capacity = cand_capacity;
    p.cand_token = cand_token;
    p.cand_score = cand_score;
    p.cand_parent = cand_parent;
    p.next_frontier_cand = next_frontier_cand;
    p.next_cum = next_cum;
    p.chunks = accept_chunks(V);
    p.chunk_elems = kArgmaxChunk;
    p.vec_ok = (aligned16(logits) && ld_logits % 4 == 0) ? 1 : 0;
    const size_t n = (size_t)B * F * p.chunks;
    char* w = (char*)workspace;
    p.part_m = (float*)w;
    w += align_up(n * sizeof(float));
    p.part_s = (float*)w;
    w += align_up(n * sizeof(float));
    p.part_tv = (float*)w;
    w += align_up(n * K * sizeof(float));
    p.part_ti = (int32_t*)w;
    return launch_draft_expand(p, (hipStream_t)stream) == hipSuccess ? VS_OK : VS_ERR_HIP;
}

int32_t vs_draft_tree_build(const int32_t* cand_token, const float* cand_score, const int32_t* cand_parent, int32_t B,
                            int32_t M, int32_t cand_capacity, int32_t N, const int32_t* root_token, int32_t* parent,
                            int32_t* draft_tokens, int32_t* node_cand, int32_t* num_nodes, int32_t* status,
                            void* stream) {
    if (!cand_token || !cand_score || !cand_parent || !parent || !draft_tokens || !node_cand || !num_nodes)
        return VS_ERR_NULL;
    if (B < 1 || M < 1 || M > kMaxDraftTotal || cand_capacity < M || N < 1 || N > VS_MAX_TREE - 1) return VS_ERR_SHAPE;
    if (const int32_t dc = check_device()) return dc;
    DraftBuildParams p{};
    p.cand_token = cand_token;
    p.cand_score = cand_score;
    p.cand_parent = cand_parent;
    p.root_token = root_token;
    p.B = B;
    p.M = M;
    p.N = N;
    p.cand_capacity = cand_capacity;
    p.parent = parent;
    p.tokens = draft_tokens;
    p.node_cand = node_cand;
    p.num_nodes = num_nodes;
    p.status = status;
    return launch_draft_tree_build(p, (hipStream_t)stream) == hipSuccess ? VS_OK : VS_ERR_HIP;
}

int32_t vs_tree_kv_commit(const vs_kv_desc* d, void* k_cache, void* v_cache, const int32_t* prefix_len,
                          const int32_t* path, const int32_t* accepted_len, int32_t* new_prefix_len,
                          int32_t* status, void* stream) {
    if (!d || !k_cache || !v_cache || !prefix_len || !path || !accepted_len || !new_prefix_len) return VS_ERR_NULL;
    if (d->B < 1 || d->T < 1 || d->T > VS_MAX_TREE || d->Hkv < 1 || d->d < 1 || d->num_layers < 1) return VS_ERR_SHAPE;
    if (d->dtype != VS_BF16 && d->dtype != VS_F32) return VS_ERR_DTYPE;
    const int64_t eb = d->dtype == VS_BF16 ? 2 : 4;
    if (d->stride_head < 0 || d->stride_tok < d->d || d->stride_layer < 0) return VS_ERR_LAYOUT;
    if (d->paged) {
        if (!is_pow2(d->block_size) || d->block_size < 16) return VS_ERR_LAYOUT;
        if (d->max_blocks < 1 || d->num_blocks < 1 || d->stride_block < 0) return VS_ERR_LAYOUT;
        if (!d->block_table) return VS_ERR_NULL;
        if (d->T > (int64_t)d->max_blocks * d->block_size) return VS_ERR_LAYOUT;
    } else {
        if (d->stride_seq < 0 || d->capacity < d->T) return VS_ERR_LAYOUT;
    }
    // rows move in 16-byte pieces
    if ((d->d * eb) % 16 || (d->stride_tok * eb) % 16 || (d->stride_head * eb) % 16 || (d->stride_layer * eb) % 16 ||
        ((d->paged ? d->stride_block : d->stride_seq) * eb) % 16)
        return VS_ERR_LAYOUT;
    if (!aligned16(k_cache) || !aligned16(v_cache)) return VS_ERR_LAYOUT;
    if (new_prefix_len == prefix_len) return VS_ERR_LAYOUT;
    if ((((int64_t)d->num_layers * 2 * d->Hkv * (d->d * eb / 16)) + 255) / 256 > 0x7fffffffLL || d->B > kMaxGridY) return VS_ERR_SHAPE;
    if (const int32_t dc = check_device()) return dc;
    CommitParams p{};
    p.k = k_cache;
    p.v = v_cache;
    p.prefix_len = prefix_len;
    p.path = path;
    p.accepted_len = accepted_len;
    p.block_table = d->paged ? d->block_table : nullptr;
    p.new_prefix_len = new_prefix_len;
    p.status = status;
    p.B = d->B;
    p.T = d->T;
    p.Hkv = d->Hkv;
    p.chunks_per_row = (int32_t)(d->d * eb / 16);
    p.items_per_seq = (int64_t)d->num_layers * 2 * d->Hkv * p.chunks_per_row;
    p.paged = d->paged ? 1 : 0;
    p.block_size = d->paged ? d->block_size : 1;
    p.block_shift = 0;
    while ((1 << p.block_shift) < p.block_size) ++p.block_shift;
    p.max_blocks = d->max_blocks;
    p.num_blocks = d->num_blocks;
    p.capacity = d->capacity;
    p.stride_layer_bytes = d->stride_layer * eb;
    p.stride_seq_bytes = d->stride_seq * eb;
    p.stride_block_bytes = d->stride_block * eb;
    p.stride_head_bytes = d->stride_head * eb;
    p.stride_tok_bytes = d->stride_tok * eb;
    return launch_kv_commit(p, (hipStream_t)stream) == hipSuccess ? VS_OK : VS_ERR_HIP;
}


} // extern "C"
