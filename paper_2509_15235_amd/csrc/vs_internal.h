// Internal declarations shared by the HIP translation units of libvispec_verify.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "vispec_verify.h"

namespace vs {

// The machine this library is written for (MI355X, gfx950): what the launch planner and the
// kernels' workgroup-id remap assume. api.hip checks the architecture of the current device
// before the first launch on it (VS_ERR_NO_DEVICE otherwise).
constexpr int kNumCUs = 256;            // compute units
constexpr int kNumXCDs = 8;             // accelerator dies; consecutive workgroup ids go round-robin over them
constexpr int kLdsBytesPerCU = 160 * 1024;
constexpr int kMaxGridY = 65535;        // largest grid extent in y and z that every HIP device takes
constexpr int64_t kMaxGridX = 0x7fffffff; // ... and in x
constexpr int kManyUnits = 48;          // (sequence, KV head) units from which the straight loop fills the CUs unaided

constexpr int kWave = 64;
constexpr int kTileKeys = 32;   // keys per MFMA score block of the attention kernel
constexpr int kIterKeys = 64;   // keys staged in LDS per loop iteration (two score blocks)
constexpr int kRowBlock = 32;   // query rows per MFMA row block
constexpr int kMaxWaves = 8;    // waves per workgroup in the MFMA attention kernel
constexpr int kArgmaxBlock = 256;
constexpr int kAcceptChunk = 4096; // floats of a logits row per workgroup of the scans: 256 threads x 4 x 16 bytes
constexpr int kBalMaxSeqs = 64;   // balanced schedule: sequences per call (a lane each)
constexpr int kBalMaxChunks = 64; // ... and shares per (KV head, row group)
constexpr int kResidentMaxKeys = 192; // keys of one split that the resident attention kernel keeps in LDS (six 32-key tiles:
                                      // with eight, its four-row-block form runs out of registers)

// Everything the attention kernels need, passed by value.
struct AttnParams {
    const void* q;
    const void* k;
    const void* v;
    void* out;
    const int32_t* prefix_len;
    const int32_t* parent;
    const uint64_t* tree_mask;  // may be null
    const int32_t* block_table; // paged only
    int32_t* status;            // may be null
    uint16_t* part_o;           // [unit][split][rows_pad][d] partial outputs, each row normalised by its own sum, bf16
    float* part_ml;             // [unit][split][rows_pad][2] running max (log2 domain), sum
    int32_t B, T, Hq, Hkv, d, group;
    int32_t tree_keys;          // T when the queries' own K/V sit behind the prefix (verification), 0 when they
                                // attend to the prefix alone (the vision adaptor's compression attention)
    int32_t rows;               // T * group: query rows per (sequence, KV head)
    int32_t rows_pad;           // rows rounded up to a multiple of kRowBlock
    int32_t max_prefix_len;
    int32_t paged, block_size, block_shift, max_blocks, num_blocks;
    int64_t capacity;
    int64_t stride_seq, stride_block, stride_head, stride_tok;
    float scale;                // softmax scale
    float scale_log2;           // softmax scale * log2(e)
    int32_t num_splits;         // grid extent over key splits
    int32_t keys_per_split;     // multiple of kIterKeys
    int32_t row_groups;
    int32_t rows_per_group;     // waves_per_group * row blocks per wave * kRowBlock
    int32_t total_wgs;          // B * Hkv * num_splits * row_groups
    int32_t* bal_table;         // balanced schedule: 64 words of workspace, the share boundaries (main kernel -> combine)
    int32_t bal_chunks;         // balanced schedule: equal shares of the batch's keys per (KV head, row group); else 0.
                                // num_splits then counts partial-result slots per KV head (shares + sequences)
};

struct AcceptParams {
    const float* logits;
    int64_t ld;
    int32_t V;
    const int32_t* draft;
    const int32_t* parent;
    int32_t B, T;
    int32_t* accepted_len;
    int32_t* path;
    int32_t* bonus;
    int32_t* row_argmax; // may be null
    int32_t* status;     // may be null
    float* part_val;     // [B*T][chunks]
    int32_t* part_idx;   // [B*T][chunks]
    int32_t chunks;
    int32_t chunk_elems; // multiple of 4
    int32_t vec_ok;      // rows are 16-byte aligned → float4 loads
};

constexpr int kMaxSampleChunks = 2048; // chunk sums of one logits row kept in LDS by the sampling walk

struct SampleParams {
    const float* logits;
    int64_t ld;
    int32_t V;
    const int32_t* draft;
    const int32_t* parent;
    const float* u_accept; // [B][T]
    const float* u_bonus;  // [B]
    int32_t B, T;
    int32_t* accepted_len;
    int32_t* path;
    int32_t* bonus;
    int32_t* status;       // may be null
    float* part_m;         // [B*T][chunks] chunk maximum of the raw logits
    float* part_s;         // [B*T][chunks] sum of 2^((l - chunk maximum) * k_log2)
    float k_log2;          // log2(e) / temperature
    int32_t chunks;
    int32_t chunk_elems;   // 4096
    int32_t vec_ok;        // rows are 16-byte aligned → float4 loads
};

constexpr int kMaxDraftK = 16;        // children per frontier node
constexpr int kMaxDraftCand = 1024;   // F * K candidates of one expansion step
constexpr int kMaxDraftTotal = 2048;  // candidates of all levels at the final selection

struct DraftExpandParams {
    const float* logits;          // [B*F][ld]
    int64_t ld;
    int32_t V;
    const float* cum_in;          // [B*F], may be null (all 0)
    const int32_t* frontier_cand; // [B*F], may be null (all -1: the root)
    int32_t B, F, K;
    int32_t cand_base, cand_capacity;
    int32_t* cand_token;          // [B][cand_capacity]
    float* cand_score;
    int32_t* cand_parent;
    int32_t* next_frontier_cand;  // [B][min(K, F*K)]
    float* next_cum;
    float* part_m;                // [B*F][chunks]
    float* part_s;
    float* part_tv;               // [B*F][chunks][K]
    int32_t* part_ti;
    int32_t chunks, chunk_elems, vec_ok;
};

struct DraftBuildParams {
    const int32_t* cand_token;    // [B][cand_capacity]
    const float* cand_score;
    const int32_t* cand_parent;
    const int32_t* root_token;    // [B], may be null
    int32_t B, M, N, cand_capacity;
    int32_t* parent;              // [B][N+1]
    int32_t* tokens;
    int32_t* node_cand;
    int32_t* num_nodes;           // [B]
    int32_t* status;              // may be null
};

struct CommitParams {
    void* k;
    void* v;
    const int32_t* prefix_len;
    const int32_t* path;         // [B][T]
    const int32_t* accepted_len; // [B]
    const int32_t* block_table;  // paged only
    int32_t* new_prefix_len;     // [B]
    int32_t* status;             // may be null
    int32_t B, T, Hkv;
    int32_t chunks_per_row;      // 16-byte pieces per row of d elements
    int64_t items_per_seq;       // layers * 2 * Hkv * chunks_per_row
    int32_t paged, block_size, block_shift, max_blocks, num_blocks;
    int64_t capacity;
    int64_t stride_layer_bytes, stride_seq_bytes, stride_block_bytes, stride_head_bytes, stride_tok_bytes;
};

// Shared tree check: returns a vs_status for lane-parallel use is in the kernels; this is
// the scalar form used on the host.
inline int32_t validate_tree_host(const int32_t* parent, int32_t T) {
    if (parent[0] != -1) return VS_STATUS_BAD_ROOT;
    for (int32_t i = 1; i < T; ++i)
        if (parent[i] < 0 || parent[i] >= i) return VS_STATUS_BAD_PARENT;
    return VS_STATUS_OK;
}

int32_t check_device(); // VS_OK when the current device is a gfx950, else VS_ERR_NO_DEVICE (api.hip)

hipError_t launch_tree_mask(const int32_t* parent, int32_t B, int32_t T, uint64_t* mask,
                            int32_t* depth, int32_t* status, hipStream_t s);
hipError_t launch_attention_generic(const AttnParams& p, int dtype, hipStream_t s);
hipError_t launch_attention_mfma(const AttnParams& p, int rpw, int waves, hipStream_t s);
bool attention_pipe_supported(int rpw, int waves);
hipError_t launch_attention_mfma_pipe(const AttnParams& p, int rpw, int waves, hipStream_t s);
bool attention_resident_supported(int row_blocks);
hipError_t launch_attention_mfma_resident(const AttnParams& p, int row_blocks, hipStream_t s);
hipError_t launch_attention_combine(const AttnParams& p, int dtype, hipStream_t s);
hipError_t launch_accept(const AcceptParams& p, hipStream_t s);
hipError_t launch_accept_sample(const SampleParams& p, hipStream_t s);
hipError_t launch_draft_expand(const DraftExpandParams& p, hipStream_t s);
hipError_t launch_draft_tree_build(const DraftBuildParams& p, hipStream_t s);
hipError_t launch_kv_commit(const CommitParams& p, hipStream_t s);

} // namespace vs
