// Tree-masked attention on the matrix cores (bf16 storage, fp32 accumulation).
//
// Math: paper Eq. 1 with a softmax scale, restricted to the keys a node may see: every
// prefix token plus the tree slots of the node's ancestor-or-self set (Section 3.1).
//
// Work decomposition. The T tree queries of the `group` query heads that share one KV
// head form rows = T * group query rows (row r -> node r / group, head r % group), so
// the contraction against that head's keys is a dense [rows x d] x [d x keys] product.
// One workgroup owns (sequence, KV head, key split, row group); each of its NW waves
// owns RPW blocks of 32 rows and keeps their queries, running softmax state and output
// accumulators in registers for the whole key range. Keys stream through double-buffered
// LDS tiles of 32 keys; the 16-byte chunks of K and V are placed so that fragment reads
// are conflict-free. Where registers allow, a tile is fetched one iteration ahead into
// registers (1 KB of consecutive memory per load instruction) and then scattered into
// LDS; the register-starved shapes use direct global-to-LDS loads instead.
//
// Per tile and row block (v_mfma_f32_32x32x16_bf16, A = 32x16, B = 16x32, C = 32x32):
//   S^T[key][row] = K[key][:] . Q[row][:]        A = K tile (LDS), B = Q (registers)
//   online softmax along keys: a lane holds 16 keys of ONE row, so the row's ancestor
//   mask, running max and running sum are plain per-lane scalars
//   O^T[d][row] += V^T[d][key] . P^T[key][row]   A = V^T (ds_read_b64_tr_b16 transposes
//   the row-major V tile on its way out of LDS), B = P (registers: the C layout of S^T
//   is, after rounding to bf16, already a B operand; the V reads pick keys in that order)
//
// With one split the normalised result is written as bf16; otherwise partials (O divided
// by the row's sum, as bf16; running max and sum as fp32) go to the workspace, laid out
// exactly as the accumulator registers are (so every store is contiguous per wave), and
// the combine kernel merges them.
#include <type_traits>

#include "attn_mfma_common.h"

namespace vs {

namespace {

template <int D, int RPW, int NW>
__global__ __launch_bounds__(NW * 64) void attn_mfma_kernel(const AttnParams p) {
    constexpr int KS = D / 16;               // k-steps of the S^T product
    constexpr int DB = D / 32;               // 32-channel blocks of the output
    // Two waves per SIMD (NW == 8) share one barrier per iteration and would otherwise sit
    // in the same stage all the time: both on the matrix core, then both on the VALU. The
    // upper half of the waves therefore runs its P.V stage one iteration late (STAGGER),
    // which needs 32-key iterations and a third LDS buffer.
    constexpr bool STAGGER = (NW == 8);
    constexpr int SUB = kTileKeys * D;       // elements per 32-key block of K (or V)
    constexpr int NSUB = STAGGER ? 1 : kIterKeys / kTileKeys;
    constexpr int ITER = NSUB * kTileKeys;   // keys per loop iteration
    constexpr int TILE = NSUB * SUB;         // elements staged per iteration for K (or V)
    constexpr int BPS = SUB * 2 / 1024;      // 1 KB direct-to-LDS load blocks per 32 keys
    constexpr int IPT = NSUB * BPS;          // ... per iteration
    constexpr int IPW = (IPT + NW - 1) / NW; // ... issued by each wave
    // Two row blocks per wave at two waves per SIMD (256 registers each) do not leave room
    // for both blocks' queries next to the accumulators: the second block's query
    // fragments then live in a lane-private LDS slot (written once, by a direct load)
    // instead of being spilled to scratch memory by the compiler.
    constexpr bool QL = (RPW == 2 && NW == 8);
    constexpr int QR0 = QL ? KS / 2 : KS;          // k-steps of row block 0 whose queries stay in registers
    constexpr int NQL = QL ? (KS - QR0) + KS : 0;  // LDS query slots (1 KB each) per wave
    // Tile copies run PD iterations ahead of their use (deeper when LDS allows: short
    // iterations do not cover the memory latency with a single tile in flight).
    constexpr int LPT = 2 * IPW;                   // load instructions per wave and tile copy
    // Direct global-to-LDS loads need no registers but are issued slowly; where registers
    // are free (no LDS-resident queries) tiles are staged through registers instead, one
    // iteration ahead.
    constexpr bool DIRECT = QL || IPW > 8 || (RPW == 2 && IPW > 4);
    // Staged copies fetch whole rows: one load instruction of a wave reads 1 KB of consecutive
    // memory (RPI tokens of D channels; lane q -> row q / LPR, 16-byte chunk q % LPR).
    constexpr int LPR = D / 8;
    constexpr int RPI = 64 / LPR;
    constexpr int PD = 1;
    constexpr int NBUF = PD + (STAGGER ? 2 : 1);
    static_assert((PD - 1) * LPT < 64, "vmcnt has six bits");

    // Tiles live in LDS in 16-byte chunks placed so that every access is conflict-free and
    // every address is "per-lane constant + immediate". A direct-to-LDS load instruction
    // writes lane q's 16 bytes at (1 KB block i) + 16 q, and each lane may fetch any chunk:
    //   K: block i, lane q holds row 16*(i / (D/32)) + q%16, chunk 4*(i % (D/32)) + q/16
    //   V: block i, lane q holds row 16*(i / (D/32)) + 4*(q/16) + (q%16)/4, chunk 4*(i % (D/32)) + q%4
    __shared__ __attribute__((aligned(1024))) uint16_t sK[NBUF][TILE];
    __shared__ __attribute__((aligned(1024))) uint16_t sV[NBUF][TILE];
    __shared__ __attribute__((aligned(1024))) uint16_t sQ[QL ? NW * NQL * 512 : 8];
    __shared__ int32_t sp[VS_MAX_TREE];
    __shared__ int32_t sflag;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // wave-uniform, lives in an SGPR
    const int half = lane >> 5;
    const int col = lane & 31;

    // Workgroup id -> (sequence, KV head, row group, split). Consecutive hardware ids go
    // round-robin over the 8 XCDs; the remap gives every XCD a contiguous range of work, so the
    // workgroups of one (sequence, KV head) share an XCD's L2 for their K/V as far as they fit,
    // and - splits being the fastest index - all key splits of a row group run on one XCD: the
    // combine workgroups of those rows, placed by the same remap, then read a slice of the
    // workspace that only this XCD has touched. Measured on one C3 layer (10 splits): 19.0 us per
    // call with row groups fastest and the combine grid in natural order, 16.7 us with both
    // kernels laid out this way; with only one of the two changed 19.4 (main) / 17.2 (combine).
    const int per_xcd = (p.total_wgs + 7) >> 3;
    const int v = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (v >= p.total_wgs) return;
    const int split = v % p.num_splits;
    int rest = v / p.num_splits;
    const int rg = rest % p.row_groups;
    rest /= p.row_groups;
    const int kvh = rest % p.Hkv;
    const int b = rest / p.Hkv;

    // With caller-supplied masks the tree was checked by the mask builder (which zeroes the
    // masks of a malformed tree); otherwise check it here.
    const int32_t S = p.prefix_len[b]; // requested before the tree is read: one latency, not two
    int32_t tree_code = VS_STATUS_OK;
    if (p.tree_mask || p.tree_keys == 0) {
        if (tid == 0) sflag = 0;
        __syncthreads();
    } else {
        tree_code = load_tree(p.parent + (int64_t)b * p.T, p.T, sp, &sflag);
    }
    const bool s_ok = prefix_ok(p, S);
    if (kvh == 0 && split == 0 && rg == 0) report_status(p, b, tree_code, s_ok, S, &sflag);
    if (tree_code != VS_STATUS_OK || !s_ok) return;

    const int nk = S + p.tree_keys;
    const int k0 = split * p.keys_per_split;
    if (k0 >= nk) return;
    const int k1 = min(nk, k0 + p.keys_per_split);

    // ---- asynchronous global -> LDS copy of one K/V tile (no registers in between).
    // Load block i covers the 16 tokens r0 .. r0+15 (r0 a multiple of 16, so one cache
    // block in paged mode) and 32 channels. Tokens past the last valid one re-read that
    // last token: finite values that the mask turns into zero weights.
    const uint16_t* kbase = (const uint16_t*)p.k;
    const uint16_t* vbase = (const uint16_t*)p.v;
    const int64_t head_base = (p.paged ? 0 : (int64_t)b * p.stride_seq) + (int64_t)kvh * p.stride_head;
    const int stride_tok = (int)p.stride_tok;           // host guarantees 32-bit lane offsets
    const int krow_l = lane & 15, kcol_l = (lane >> 4) * 8;
    const int vrow_l = 4 * (lane >> 4) + ((lane & 15) >> 2), vcol_l = (lane & 3) * 8;
    // Register path: where chunk c (16 bytes) of row r of a 32-key block lives in LDS. Same
    // placement as above except that K rows are XOR-swizzled by 4*(c%4), which turns the
    // 16-way bank conflict of writing one row's chunks into a 4-way one and leaves the
    // fragment reads (16 rows at one chunk) conflict-free:
    //   K: ((r/16)*DB + c/4) * 1024 + (c%4) * 256 + ((r%16) ^ 4*(c%4)) * 16
    //   V: ((r/16)*DB + c/4) * 1024 + (4*(r%16) + c%4) * 16
    const int lrow = lane / LPR, lchunk = lane % LPR;
    u32x4 kreg[DIRECT ? 1 : IPW], vreg[DIRECT ? 1 : IPW]; // staged tile (register path)
    uint32_t k_st[DIRECT ? 1 : IPW], v_st[DIRECT ? 1 : IPW]; // LDS byte offsets inside one buffer
    if constexpr (!DIRECT) {
#pragma unroll
        for (int j = 0; j < IPW; ++j) {
            const int i = wave * IPW + j;
            const int r = (i % BPS) * RPI + lrow, c = lchunk;
            k_st[j] = (uint32_t)((i / BPS) * (SUB * 2) + ((r >> 4) * DB + (c >> 2)) * 1024 + (c & 3) * 256 +
                                 (((r & 15) ^ (4 * (c & 3))) * 16));
            v_st[j] = (uint32_t)((i / BPS) * (SUB * 2) + ((r >> 4) * DB + (c >> 2)) * 1024 + (4 * (r & 15) + (c & 3)) * 16);
        }
    }
    auto fetch = [&](int kt, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < IPW; ++j) {
            const int i = wave * IPW + j; // block index, uniform per wave
            if (i < IPT) {
                if constexpr (DIRECT) {
                    const int r0 = kt + kTileKeys * (i / BPS) + 16 * ((i % BPS) / DB);
                    const int c0 = 32 * (i % DB);
                    int ktok = min(r0 + krow_l, k1 - 1), vtok = min(r0 + vrow_l, k1 - 1);
                    int64_t base = head_base;
                    if (p.paged) {
                        int32_t blk = p.block_table[(int64_t)b * p.max_blocks + (min(r0, k1 - 1) >> p.block_shift)];
                        if ((uint32_t)blk >= (uint32_t)p.num_blocks) blk = 0; // reported through status
                        base += (int64_t)blk * p.stride_block;
                        ktok &= p.block_size - 1;
                        vtok &= p.block_size - 1;
                    }
                    const uint32_t koff = (uint32_t)(ktok * stride_tok + c0 + kcol_l);
                    const uint32_t voff = (uint32_t)(vtok * stride_tok + c0 + vcol_l);
                    __builtin_amdgcn_global_load_lds(kbase + base + koff, (lds_void*)(sK[buf] + i * 512), 16, 0, 0);
                    __builtin_amdgcn_global_load_lds(vbase + base + voff, (lds_void*)(sV[buf] + i * 512), 16, 0, 0);
                } else {
                    const int r0 = kt + kTileKeys * (i / BPS) + RPI * (i % BPS); // RPI divides 16: one page
                    int tok = min(r0 + lrow, k1 - 1);
                    int64_t base = head_base;
                    if (p.paged) {
                        int32_t blk = p.block_table[(int64_t)b * p.max_blocks + (min(r0, k1 - 1) >> p.block_shift)];
                        if ((uint32_t)blk >= (uint32_t)p.num_blocks) blk = 0; // reported through status
                        base += (int64_t)blk * p.stride_block;
                        tok &= p.block_size - 1;
                    }
                    const uint32_t off = (uint32_t)(tok * stride_tok + lchunk * 8);
                    kreg[j] = *(const u32x4*)(kbase + base + off);
                    vreg[j] = *(const u32x4*)(vbase + base + off);
                }
            }
        }
    };
    // register path: write the staged tile into LDS buffer `buf`
    auto stash = [&](int buf) __attribute__((always_inline)) {
        if constexpr (!DIRECT) {
#pragma unroll
            for (int j = 0; j < IPW; ++j) {
                const int i = wave * IPW + j;
                if (i < IPT) {
                    *(u32x4*)((char*)sK[buf] + k_st[j]) = kreg[j];
                    *(u32x4*)((char*)sV[buf] + v_st[j]) = vreg[j];
                }
            }
        }
    };
    fetch(k0, 0); // in flight while the queries are loaded; tokens past the end are clamped

    // ---- this wave's rows, their masks and queries
    const int row_base = rg * p.rows_per_group + wave * (RPW * kRowBlock);
    const bool wave_active = row_base < p.rows;
    uint64_t mask[RPW];
    bf16x8 qf[RPW][KS];
    const uint16_t* qbase = (const uint16_t*)p.q;
#pragma unroll
    for (int rb = 0; rb < RPW; ++rb) {
        // rows past the end repeat the last row (finite data, results discarded)
        const int r = min(row_base + rb * kRowBlock + col, p.rows - 1);
        const int node = r / p.group;
        const int hq = kvh * p.group + (r - node * p.group);
        mask[rb] = p.tree_keys == 0 ? 0ull : (p.tree_mask ? p.tree_mask[(int64_t)b * p.T + node] : ancestor_mask(sp, node));
        const uint16_t* qr = qbase + (((int64_t)b * p.T + node) * p.Hq + hq) * D + half * 8;
        if (wave_active) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (QL && (rb == 1 || ks >= QR0)) {
                    const int slot = rb == 1 ? (KS - QR0) + ks : ks - QR0;
                    __builtin_amdgcn_global_load_lds(qr + ks * 16, (lds_void*)(sQ + (wave * NQL + slot) * 512), 16, 0, 0);
                } else {
                    qf[rb][ks] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qr + ks * 16));
                }
            }
        }
    }

    float m2[RPW], lsum[RPW]; // running max (log2 domain, scaled) and this lane's share of the sum
    f32x16 acc[RPW][DB];
#pragma unroll
    for (int rb = 0; rb < RPW; ++rb) {
        m2[rb] = -INFINITY;
        lsum[rb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][db][r] = 0.f;
    }

    // per-lane LDS offsets (elements); everything else is a compile-time immediate
    // K fragment of k-step ks (chunk 2*ks + half of row `col`): k_lane[ks & 1] + ks*256
    const int kx0 = DIRECT ? 0 : 4 * half, kx1 = DIRECT ? 0 : 8 + 4 * half;
    const int k_lane[2] = {(col >> 4) * (DB * 512) + half * 128 + ((col & 15) ^ kx0) * 8,
                           (col >> 4) * (DB * 512) + half * 128 + ((col & 15) ^ kx1) * 8};
    const int t16 = lane & 15;                                               // transposing V read: 16-lane groups
    const int v_lane = half * 128 + (t16 >> 2) * 32 + ((lane >> 4) & 1) * 16 + ((t16 >> 1) & 1) * 8 + (t16 & 1) * 4;
    //                 + sl*(DB*512) + db*512 + u*256
    const uint16_t* q_lane = sQ + wave * (NQL * 512) + lane * 8;             // + slot*512

    // Stage 1 of a 32-key tile for this wave's row blocks: scores, mask, online softmax,
    // probabilities as MFMA operands in pf. MASKED tiles hold tree slots or the end of the
    // key range; all others are pure prefix and skip the visibility logic.
    bf16x8 pf[RPW][2];
    auto score = [&](auto masked_tag, int kt, const uint16_t* kblock) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        const uint16_t* tK[2] = {kblock + k_lane[0], kblock + k_lane[1]};
        // ---- per row block: S^T = K . Q^T, mask, online softmax, P as a B operand.
        // Lane (col, half) holds keys 8*(r/4) + 4*half + r%4 of row `col`.
        // Each K fragment is read from LDS once and feeds every row block. The reads run
        // PF k-steps ahead of the MFMAs that consume them (software pipeline; the
        // scheduling barriers keep the compiler from serialising read -> wait -> MFMA).
        constexpr int PF = 2;
        f32x16 sc[RPW];
#pragma unroll
        for (int rb = 0; rb < RPW; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) sc[rb][r] = 0.f;
        u32x4 ka[PF + 1], qa[PF + 1][RPW]; // fragment ring buffers (only LDS-resident queries use qa)
        auto load_frags = [&](int ks) __attribute__((always_inline)) {
            ka[ks % (PF + 1)] = *(const u32x4*)(tK[ks & 1] + ks * 256);
#pragma unroll
            for (int rb = 0; rb < RPW; ++rb) {
                if (QL && (rb == 1 || ks >= QR0)) {
                    const int slot = rb == 1 ? (KS - QR0) + ks : ks - QR0;
                    qa[ks % (PF + 1)][rb] = *(const u32x4*)(q_lane + slot * 512);
                }
            }
        };
#pragma unroll
        for (int ks = 0; ks < PF; ++ks) load_frags(ks);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks + PF < KS) load_frags(ks + PF);
            __builtin_amdgcn_sched_barrier(0);
            const bf16x8 a = __builtin_bit_cast(bf16x8, ka[ks % (PF + 1)]);
#pragma unroll
            for (int rb = 0; rb < RPW; ++rb) {
                const bf16x8 bq = (QL && (rb == 1 || ks >= QR0)) ? __builtin_bit_cast(bf16x8, qa[ks % (PF + 1)][rb])
                                                                  : qf[rb][ks];
                sc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bq, sc[rb], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int rb = 0; rb < RPW; ++rb) {
            f32x16& s = sc[rb];
            if constexpr (MASKED) {
                const int rel = kt + 4 * half - S; // tree slot of this lane's key 0 (negative: prefix)
                const uint32_t tree_end = (uint32_t)(k1 - S);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int sh = rel + 8 * (r >> 2) + (r & 3);
                    const uint32_t bit = (uint32_t)(mask[rb] >> (sh & 63)) & 1u;
                    const bool vis = (sh < 0) | (((uint32_t)sh < tree_end) & (bit != 0));
                    s[r] = vis ? s[r] : -INFINITY;
                }
            }
            float mx = fmaxf(fmaxf(s[0], s[1]), s[2]);
#pragma unroll
            for (int r = 3; r < 15; r += 2) mx = fmaxf(fmaxf(mx, s[r]), s[r + 1]);
            mx = fmaxf(mx, s[15]);
            mx = half_max(mx);
            // Lazy reference maximum: m2 only moves when the tile's maximum exceeds it by more
            // than kLazy (2^8 in the linear domain). Probabilities then reach at most 2^8,
            // well inside bf16/fp32 range, the result is unchanged (numerator and denominator
            // share the reference), and the accumulator rescale below becomes rare.
            const float mt = mx * p.scale_log2;
            const float m_new = (mt > m2[rb] + kLazy) ? mt : m2[rb];
            const float m_use = (MASKED && m_new == -INFINITY) ? 0.f : m_new; // no visible key yet
            const float alpha = __builtin_amdgcn_exp2f(m2[rb] - m_use);
            m2[rb] = m_new;
            float psum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                s[r] = __builtin_amdgcn_exp2f(fmaf(s[r], p.scale_log2, -m_use)); // exp2(-inf) = 0
                psum += s[r];
            }
            lsum[rb] = lsum[rb] * alpha + psum;
            if (__any(alpha != 1.f)) {
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[rb][db][r] *= alpha;
            }
#pragma unroll
            for (int sl = 0; sl < 2; ++sl) {
                u32x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const f32x2 pr = {s[8 * sl + 2 * e], s[8 * sl + 2 * e + 1]};
                    w[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
                }
                pf[rb][sl] = __builtin_bit_cast(bf16x8, w);
            }
        }

    };
    // Stage 2: O^T += V^T . P^T. The A operand (channel `col` of block db, keys in the
    // order P holds them) comes from two transposing reads of 4 keys x 16 channels.
    auto pv = [&](const uint16_t* vblock) __attribute__((always_inline)) {
        const uint16_t* tV = vblock + v_lane;
        constexpr int NV = 2 * DB; // V^T fragments per 32 keys, step = sl * DB + db
        constexpr int PF = 2;
        s16x4 va[PF + 1][2];
        auto load_v = [&](int st) __attribute__((always_inline)) {
            const int sl = st / DB, db = st % DB;
            va[st % (PF + 1)][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tV + sl * (DB * 512) + db * 512));
            va[st % (PF + 1)][1] =
                __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tV + sl * (DB * 512) + db * 512 + 256));
        };
#pragma unroll
        for (int st = 0; st < PF; ++st) load_v(st);
#pragma unroll
        for (int st = 0; st < NV; ++st) {
            if (st + PF < NV) load_v(st + PF);
            __builtin_amdgcn_sched_barrier(0);
            const int sl = st / DB, db = st % DB;
            const bf16x8 a = __builtin_bit_cast(
                bf16x8, __builtin_shufflevector(va[st % (PF + 1)][0], va[st % (PF + 1)][1], 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
            for (int rb = 0; rb < RPW; ++rb)
                acc[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[rb][sl], acc[rb][db], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // the other tiles of the prefetch window; then wait for tile 0, the queries and masks
#pragma unroll
    for (int t = 1; t < PD; ++t) fetch(k0 + t * ITER, t);
    __builtin_amdgcn_s_waitcnt(wait_vm((PD - 1) * LPT));
    stash(0);
    __syncthreads();

    // Iterations whose keys end at or before min(S, k1) are pure prefix; the rest take the
    // masked path.
    const int k_plain = k0 + max(0, (min(S, k1) - k0) / ITER) * ITER;
    int buf = 0, prv = 0;
    int kt = k0;
    // One iteration: start the next keys' copy into a buffer nobody reads any more, do this
    // wave's stages, then wait until the copy has landed and every wave is done.
    auto step = [&](auto late_tag, auto masked_tag) __attribute__((always_inline)) {
        constexpr bool LATE = decltype(late_tag)::value;
        const int nxt = (buf + 1 == NBUF) ? 0 : buf + 1;
        // copy the tile PD iterations ahead into a buffer whose readers are all done; issued
        // even past the end of the range (clamped tokens) so that every wave always has the
        // same number of loads in flight and the counted wait below stays exact
        if (PD > 1 || kt + ITER < k1) fetch(kt + PD * ITER, (buf + PD) % NBUF);
        if (wave_active) {
            if constexpr (LATE) {
                if (kt > k0) pv(sV[prv]); // previous iteration's probabilities, kept in pf
                score(masked_tag, kt, sK[buf]);
            } else {
#pragma unroll
                for (int sub = 0; sub < NSUB; ++sub) {
                    if (sub == 0 || kt + sub * kTileKeys < k1) {
                        score(masked_tag, kt + sub * kTileKeys, sK[buf] + sub * SUB);
                        pv(sV[buf] + sub * SUB);
                    }
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(wait_vm((PD - 1) * LPT)); // the next tile has arrived
        stash(nxt);
        __syncthreads();
        prv = buf;
        buf = nxt;
    };
    if (STAGGER && wave >= NW / 2) {
        for (; kt < k_plain; kt += ITER) step(std::true_type{}, std::false_type{});
        for (; kt < k1; kt += ITER) step(std::true_type{}, std::true_type{});
        if (wave_active) pv(sV[prv]);
    } else {
        for (; kt < k_plain; kt += ITER) step(std::false_type{}, std::false_type{});
        for (; kt < k1; kt += ITER) step(std::false_type{}, std::true_type{});
    }

    if (!wave_active) return;

    // ---- epilogue: lane (col, half) holds, for row `col`, channels db*32 + 8*(r/4) + 4*half + r%4
#pragma unroll
    for (int rb = 0; rb < RPW; ++rb) {
        const int r_local = row_base + rb * kRowBlock + col;
        const float l = half_sum(lsum[rb]);
        if (p.num_splits == 1) {
            if (r_local >= p.rows) continue;
            const int node = r_local / p.group;
            const int hq = kvh * p.group + (r_local - node * p.group);
            uint16_t* o = (uint16_t*)p.out + (((int64_t)b * p.T + node) * p.Hq + hq) * D;
            const float inv = 1.f / l;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    u32x2 w;
                    w[0] = pack_bf16x2(acc[rb][db][4 * q4] * inv, acc[rb][db][4 * q4 + 1] * inv);
                    w[1] = pack_bf16x2(acc[rb][db][4 * q4 + 2] * inv, acc[rb][db][4 * q4 + 3] * inv);
                    *(u32x2*)(o + db * 32 + 8 * q4 + 4 * half) = w;
                }
        } else {
            if (row_base + rb * kRowBlock >= p.rows) continue; // whole block is padding
            const int64_t blk = part_block(p, (int64_t)b * p.Hkv + kvh, split, (row_base >> 5) + rb);
            uint16_t* po = p.part_o + blk * (kRowBlock * D);
            const float inv = l > 0.f ? 1.f / l : 0.f; // no visible key in this split: zeros, weight 0
#pragma unroll
            for (int db = 0; db < DB; ++db) store_partial<D>(po, db, lane, acc[rb][db], inv);
            if (half == 0) {
                const f32x2 ml = {m2[rb], l};
                const int64_t mlb = ml_block(p, (int64_t)b * p.Hkv + kvh, split, (row_base >> 5) + rb);
                *(f32x2*)(p.part_ml + (mlb + col) * 2) = ml;
            }
        }
    }
}

// Merges the key splits: out = sum_s w_s (O_s / l_s) / sum_s w_s with w_s = 2^(m_s - M) l_s per query row
// (the main kernels store O_s / l_s, see pack_partial).
// One wave per (sequence, KV head, 32-row block, 32-channel block); lanes map to the
// partials exactly as the accumulator registers did, the result is transposed through LDS
// so that the bf16 rows leave as 16-byte stores. The kernel is pure latency, so the prefix
// length, every split's (max, sum) and every split's partials are requested back to back
// before anything is waited for (splits past the sequence's end hold stale workspace
// bytes; they are loaded but never used). A sequence whose prefix length is out of range
// is skipped; a malformed tree (reported by the main kernel) leaves unspecified output.
constexpr int kCombineBatch = 16; // splits whose partials are in flight together
template <int D, bool BAL>
__global__ __launch_bounds__(kWave) void attn_combine_kernel(const AttnParams p) {
    constexpr int DB = D / 32;
    // partials in flight together. A sequence of the balanced schedule has a handful of pieces: a small
    // batch keeps the kernel at eight waves per SIMD, which its thousands of one-wave workgroups need.
    constexpr int BATCH = BAL ? 4 : kCombineBatch;
    __shared__ __attribute__((aligned(16))) uint16_t so[kRowBlock][32 + 8];
    __shared__ int32_t sslot[BAL ? kBalMaxChunks : 1]; // balanced schedule: the slots of this sequence's pieces
    // Workgroup id -> (unit, row group, row block of the group, channel block), in contiguous ranges
    // per XCD like the main kernels: with splits as the main kernels' fastest index, the partials of
    // a row group were all written by one XCD, and that is the XCD these rows' combine workgroups
    // land on. Every XCD then stays on its own eighth of the workspace in both kernels and from one
    // call to the next (2.3 us per one-layer call against a grid whose neighbouring workgroups -
    // on eight different XCDs - read neighbouring pieces of the same partial blocks; the counters
    // show the partials still arrive from memory, not from L2, so what is saved is address
    // translation and fabric traffic rather than the fetch itself).
    const int rbg = p.rows_per_group / kRowBlock; // row blocks per row group
    const int items = p.B * p.Hkv * p.row_groups * rbg * DB;
    const int per_xcd = (items + 7) >> 3;
    const int vi = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (vi >= items) return;
    const int db = vi % DB;
    int rest = vi / DB;
    const int rbk = (rest / rbg % p.row_groups) * rbg + rest % rbg;
    const int unit = rest / (rbg * p.row_groups);
    if (rbk * kRowBlock >= p.rows) return; // padding of the last row group
    const int b = unit / p.Hkv, kvh = unit % p.Hkv;
    const int lane = threadIdx.x, col = lane & 31, half = lane >> 5;
    const int32_t S = BAL ? 0 : p.prefix_len[b];
    const int64_t punit = BAL ? kvh : unit; // whose partial-result slots these are
    const f32x2* gml = (const f32x2*)p.part_ml + ml_block(p, punit, 0, rbk) + col; // + slot * kRowBlock
    const int64_t blk0 = part_block(p, punit, 0, rbk);
    const int64_t blk_stride = p.rows_pad / kRowBlock; // blocks per slot
    const uint16_t* po0 = p.part_o + blk0 * (kRowBlock * D) + ((db * 2) * 64 + lane) * 8;

    float den = 0.f, M = -INFINITY;
    f32x4 num[4];
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) num[q4] = f32x4{0.f, 0.f, 0.f, 0.f};
    int nsplit = 0;
    int nload = p.num_splits; // partials requested (splits past the sequence's end included: they are not used)
    if constexpr (BAL) {
        // the shares that hold keys of this sequence, found the way the main kernel found them
        int start, steps, total;
        bool usable;
        bal_scan(p, lane, start, steps, total, usable);
        const int bounds = p.bal_table[lane];
        const int up = __shfl_down(bounds, 1);
        const int hi = lane + 1 < p.bal_chunks ? up : total;
        const int s0 = __builtin_amdgcn_readlane(start, b), t = __builtin_amdgcn_readlane(steps, b);
        int t0, t1;
        const bool mine = lane < p.bal_chunks && bal_piece(bounds, hi, s0, t, t0, t1);
        const uint64_t m = __ballot(mine);
        nsplit = __popcll(m);
        if (nsplit <= 1) return; // no usable prefix, or a single piece: its rows are final already
        if (mine) sslot[__popcll(m & ((1ull << lane) - 1ull))] = lane + b;
        __syncthreads();
        nload = nsplit;
    }
    auto slot_of = [&](int u) __attribute__((always_inline)) { return BAL ? sslot[u] : u; };
    for (int s0 = 0; s0 < nload; s0 += BATCH) {
        f32x2 ml[BATCH];
        u32x4 o[BATCH][2];
#pragma unroll
        for (int u = 0; u < BATCH; ++u)
            if (s0 + u < nload) ml[u] = __builtin_nontemporal_load(gml + slot_of(s0 + u) * kRowBlock);
#pragma unroll
        for (int u = 0; u < BATCH; ++u)
            if (s0 + u < nload) {
                const uint16_t* po = po0 + slot_of(s0 + u) * blk_stride * (kRowBlock * D);
#pragma unroll
                for (int hp = 0; hp < 2; ++hp) o[u][hp] = __builtin_nontemporal_load((const u32x4*)(po + hp * 512));
            }
        if (!BAL && s0 == 0) {
            if (!prefix_ok(p, S)) return;
            nsplit = min(p.num_splits, (S + p.tree_keys + p.keys_per_split - 1) / p.keys_per_split);
        }
        // this batch's maximum joins the running one; what was summed so far is rescaled
        float Mb = M;
#pragma unroll
        for (int u = 0; u < BATCH; ++u)
            if (s0 + u < nsplit) Mb = fmaxf(Mb, ml[u][0]);
        const float resc = (M == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(M - Mb); // nothing summed yet: 0
        den *= resc;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) num[q4] *= resc;
        M = Mb;
#pragma unroll
        for (int u = 0; u < BATCH; ++u)
            if (s0 + u < nsplit) { // uniform
                // a split that saw no visible key for the row has max -inf, sum 0 and zero partials
                // the split's row is stored normalised: its weight is 2^(m_s - M) * l_s
                const float w = (ml[u][0] != -INFINITY) ? __builtin_amdgcn_exp2f(ml[u][0] - M) * ml[u][1] : 0.f;
                den += w;
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const u32x2 piece = {o[u][q4 >> 1][2 * (q4 & 1)], o[u][q4 >> 1][2 * (q4 & 1) + 1]};
                    num[q4] += w * unpack_partial(piece);
                }
            }
    }
    const float inv = 1.f / den;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
        u32x2 w;
        w[0] = pack_bf16x2(num[q4][0] * inv, num[q4][1] * inv);
        w[1] = pack_bf16x2(num[q4][2] * inv, num[q4][3] * inv);
        *(u32x2*)&so[col][8 * q4 + 4 * half] = w;
    }
    __syncthreads();
    uint16_t* out = (uint16_t*)p.out;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int rl = i * 16 + (lane >> 2), ch = lane & 3;
        const int row = rbk * kRowBlock + rl;
        if (row < p.rows) {
            const int node = row / p.group;
            const int hq = kvh * p.group + (row - node * p.group);
            *(u32x4*)(out + (((int64_t)b * p.T + node) * p.Hq + hq) * D + db * 32 + ch * 8) = *(const u32x4*)&so[rl][ch * 8];
        }
    }
}

template <int D, int RPW>
hipError_t launch_nw(const AttnParams& p, int waves, hipStream_t s) {
    const dim3 grid(((p.total_wgs + 7) / 8) * 8);
    switch (waves) {
    case 1: hipLaunchKernelGGL((attn_mfma_kernel<D, RPW, 1>), grid, dim3(64), 0, s, p); break;
    case 2: hipLaunchKernelGGL((attn_mfma_kernel<D, RPW, 2>), grid, dim3(128), 0, s, p); break;
    case 4: hipLaunchKernelGGL((attn_mfma_kernel<D, RPW, 4>), grid, dim3(256), 0, s, p); break;
    case 8: hipLaunchKernelGGL((attn_mfma_kernel<D, RPW, 8>), grid, dim3(512), 0, s, p); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

} // namespace

hipError_t launch_attention_mfma(const AttnParams& p, int rpw, int waves, hipStream_t s) {
    if (p.d == 128) return rpw == 2 ? launch_nw<128, 2>(p, waves, s) : launch_nw<128, 1>(p, waves, s);
    if (p.d == 64) return rpw == 2 ? launch_nw<64, 2>(p, waves, s) : launch_nw<64, 1>(p, waves, s);
    return hipErrorInvalidValue;
}

hipError_t launch_attention_combine(const AttnParams& p, int dtype, hipStream_t s) {
    (void)dtype;
    const int items = p.B * p.Hkv * p.row_groups * (p.rows_per_group / kRowBlock) * (p.d / 32);
    const dim3 grid((unsigned)((items + 7) / 8 * 8));
    if (p.bal_chunks > 0) {
        if (p.d == 128) hipLaunchKernelGGL((attn_combine_kernel<128, true>), grid, dim3(kWave), 0, s, p);
        else if (p.d == 64) hipLaunchKernelGGL((attn_combine_kernel<64, true>), grid, dim3(kWave), 0, s, p);
        else return hipErrorInvalidValue;
    } else if (p.d == 128) hipLaunchKernelGGL((attn_combine_kernel<128, false>), grid, dim3(kWave), 0, s, p);
    else if (p.d == 64) hipLaunchKernelGGL((attn_combine_kernel<64, false>), grid, dim3(kWave), 0, s, p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

} // namespace vs
