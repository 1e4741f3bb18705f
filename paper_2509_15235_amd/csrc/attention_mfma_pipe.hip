// Tree-masked attention on the matrix cores, software-pipelined across key tiles.
//
// Same math, work decomposition, LDS chunk placement and partial-result layout as the
// kernel in attention_mfma.hip (paper Eq. 1 restricted by tree ancestry, Section 3.1).
// The difference is the schedule. Per 32-key tile t a wave has three pieces of work:
//   S(t)  = K(t) . Q^T            8 MFMAs per row block
//   P(t)  = online softmax of S(t) on the vector ALU (exp2, running max and sum, bf16)
//   O    += V(t)^T . P(t)^T       8 MFMAs per row block
// S -> P -> O of one tile depend on each other, so a straight loop leaves the matrix
// core idle during P and the vector ALU idle during S and O. Here the step for tile t
// issues S(t+1) and O(t-1) together with P(t): the sixteen MFMAs have no operand in
// common with the softmax of the same step and the hardware runs them side by side.
// One loop iteration covers two tiles (so the roles of the two score / probability
// register sets are fixed at compile time) and ends in the only barrier. Inside a step
// the instruction stream is written slot by slot - one MFMA, the LDS read of a fragment
// two slots ahead, one sixteenth of the softmax - and K and V^T fragments alternate so
// that consecutive MFMAs never share an accumulator.
//
// K/V tiles travel global -> registers -> LDS, 1 KB of consecutive memory per load
// instruction. Copies are grouped per iteration (two K tiles, two V tiles); a group is
// requested two iterations before the one that writes it to LDS in its middle, so two
// groups are in flight in two register sets. K tiles reach LDS three to four tiles ahead
// of their S step, V tiles one to two ahead of their O step, in two four-slot rings
// (tile t lives in slot t % 4).
//
// Measured on MI355X with N(0,1) inputs the loop sustains about 0.6 PFLOP/s; a loop of
// nothing but these MFMAs on random operands reaches 1.76 PFLOP/s on this machine (2.27
// on constant operands: the clock is power-managed), so the remaining gap is barrier skew,
// copy issue and the two general iterations at either end of the key range.
#include <type_traits>

#include "attn_mfma_common.h"

namespace vs {

namespace {

template <int D, int RPW, int NW, bool PAGED, bool BAL>
__global__ __launch_bounds__(NW * 64, 2) void attn_mfma_pipe_kernel(const AttnParams p) {
    constexpr int KS = D / 16;                 // k-steps of the S^T product
    constexpr int DB = D / 32;                 // 32-channel blocks of the output
    constexpr int SUB = kTileKeys * D;         // elements per 32-key tile of K (or V)
    constexpr int BPS = SUB * 2 / 1024;        // 1 KB blocks (16 keys x 32 channels) per tile
    constexpr int BPW = (BPS + NW - 1) / NW;   // ... copied by each wave
    constexpr int NSLOT = 4;

    __shared__ __attribute__((aligned(1024))) uint16_t sK[NSLOT][SUB];
    __shared__ __attribute__((aligned(1024))) uint16_t sV[NSLOT][SUB];
    __shared__ int32_t sp[VS_MAX_TREE];
    __shared__ int32_t sflag;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5;
    const int col = lane & 31;

    // One piece of work: the rows of row group `rg` of (sequence b, KV head kvh) against the keys
    // [k0, k0 + klen) of that sequence (k0 lies inside the cache). `whole`: no other piece shares these
    // rows, they leave as final output; else as the partial result of slot `slot`.
    auto run_piece = [&](const int b, const int kvh, const int rg, const int k0, const int klen, const int slot,
                         const bool whole) __attribute__((always_inline)) {
    const int32_t S = p.prefix_len[b]; // requested first, needed last: the first tiles and the queries are requested before it arrives

    // ---- tile copies. One load instruction of a wave fetches 1 KB of consecutive memory:
    // RPI whole rows (tokens) of D channels, lane q -> row q / LPR, 16-byte chunk q % LPR, so
    // every touched cache line is used completely. The 16-byte chunks are then scattered into
    // LDS so that the fragment reads are conflict-free; chunk c of tile row r lives at byte
    //   K: ((r/16)*DB + c/4) * 1024 + (c%4) * 256 + ((r%16) ^ 4*(c%4)) * 16
    //   V: ((r/16)*DB + c/4) * 1024 + (4*(r%16) + c%4) * 16
    // (the XOR spreads the chunks of one K row over the banks: 4-way instead of 16-way write
    // conflicts; reads of 16 rows at one chunk stay a permutation of 16 consecutive slots).
    // Tokens past the last valid one re-read that token (finite values that get zero weight).
    constexpr int LPR = D / 8;        // lanes (16-byte chunks) per row
    constexpr int RPI = 64 / LPR;     // rows per load instruction
    static_assert(BPS * RPI == kTileKeys, "a tile is BPS blocks of RPI rows");
    const uint16_t* kbase = (const uint16_t*)p.k;
    const uint16_t* vbase = (const uint16_t*)p.v;
    const int64_t head_base = (PAGED ? 0 : (int64_t)b * p.stride_seq) + (int64_t)kvh * p.stride_head;
    const int stride_tok = (int)p.stride_tok; // host guarantees 32-bit lane offsets
    const int lrow = lane / LPR, lchunk = lane % LPR;
    const uint32_t lane_off = (uint32_t)(lrow * stride_tok + lchunk * 8) * 2u; // bytes
    uint32_t k_st[BPW], v_st[BPW]; // this lane's LDS byte offsets inside a tile slot, per block
#pragma unroll
    for (int j = 0; j < BPW; ++j) {
        const int r = (wave * BPW + j) * RPI + lrow, c = lchunk;
        k_st[j] = (uint32_t)(((r >> 4) * DB + (c >> 2)) * 1024 + (c & 3) * 256 + (((r & 15) ^ (4 * (c & 3))) * 16));
        v_st[j] = (uint32_t)(((r >> 4) * DB + (c >> 2)) * 1024 + (4 * (r & 15) + (c & 3)) * 16);
    }
    u32x4 stage[2][4][BPW];
    // The first four tiles - K(0), K(1), K(2), V(0), through register set 1 - are requested before
    // the prefix length is known: clamped to the cache instead of the sequence, and rows that
    // turn out to lie past the sequence's last key are zeroed when the tiles go into LDS
    // (whatever the cache holds there, NaN included, must not meet a zero probability).
    {
        const int64_t cache_tokens = PAGED ? (int64_t)p.max_blocks * p.block_size : p.capacity;
        const int kend = (int)(cache_tokens < (int64_t)k0 + klen ? cache_tokens : (int64_t)k0 + klen);
        auto load_tile_early = [&](auto is_v, int t, u32x4(&r)[BPW]) __attribute__((always_inline)) {
            const uint16_t* gbase = decltype(is_v)::value ? vbase : kbase;
#pragma unroll
            for (int j = 0; j < BPW; ++j) {
                const int i = wave * BPW + j;
                if (NW * BPW == BPS || i < BPS) {
                    const int r0 = min(k0 + t * kTileKeys + RPI * i, kend - 1); // RPI divides 16: one cache block in paged mode
                    int tok = min(r0 + lrow, kend - 1);
                    int64_t base = head_base;
                    if (PAGED) {
                        int32_t blk = p.block_table[(int64_t)b * p.max_blocks + (r0 >> p.block_shift)];
                        if ((uint32_t)blk >= (uint32_t)p.num_blocks) blk = 0; // reported through status
                        base += (int64_t)blk * p.stride_block;
                        tok &= p.block_size - 1;
                    }
                    r[j] = *(const u32x4*)(gbase + base + (uint32_t)(tok * stride_tok + lchunk * 8));
                }
            }
        };
        load_tile_early(std::false_type{}, 0, stage[1][0]);
        load_tile_early(std::false_type{}, 1, stage[1][1]);
        load_tile_early(std::false_type{}, 2, stage[1][2]);
        load_tile_early(std::true_type{}, 0, stage[1][3]);
    }

    // ---- this wave's rows and queries (in flight together with the first tiles)
    const int row_base = rg * p.rows_per_group + wave * (RPW * kRowBlock);
    const bool wave_active = row_base < p.rows;
    bf16x8 qf[RPW][KS];
    int node_of[RPW];
#pragma unroll
    for (int rb = 0; rb < RPW; ++rb) {
        // rows past the end repeat the last row (finite data, results discarded)
        const int r = min(row_base + rb * kRowBlock + col, p.rows - 1);
        const int node = r / p.group;
        const int hq = kvh * p.group + (r - node * p.group);
        node_of[rb] = node;
        const uint16_t* qr = (const uint16_t*)p.q + (((int64_t)b * p.T + node) * p.Hq + hq) * D + half * 8;
        if (wave_active) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) qf[rb][ks] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qr + ks * 16));
        }
    }

    int32_t tree_code = VS_STATUS_OK;
    if (p.tree_mask || p.tree_keys == 0) {
        if (tid == 0) sflag = 0;
        __syncthreads();
    } else {
        tree_code = load_tree(p.parent + (int64_t)b * p.T, p.T, sp, &sflag);
    }
    const bool s_ok = prefix_ok(p, S);
    if (kvh == 0 && k0 == 0 && rg == 0) report_status(p, b, tree_code, s_ok, S, &sflag);
    if (tree_code != VS_STATUS_OK || !s_ok) return;

    const int nk = S + p.tree_keys;
    if (k0 >= nk) return;
    const int k1 = min(nk, k0 + klen);
    const int n = (k1 - k0 + kTileKeys - 1) / kTileKeys; // tiles of this split

    const int n_full = (k1 - k0) / kTileKeys; // tiles without a ragged end
    // first key of the split in this (sequence, KV head) slice; only used when not paged
    const char* kfast = (const char*)(kbase + head_base + (int64_t)k0 * stride_tok);
    const char* vfast = (const char*)(vbase + head_base + (int64_t)k0 * stride_tok);
    // LFAST: a full tile, so the address is a wave-uniform base plus a per-lane constant and nothing
    // needs clamping.
    // Paged caches: the block ids of the tiles to come sit one per lane in two registers (a window of
    // 128 consecutive table entries, fetched with two coalesced loads and moved along as the tiles
    // advance), so a tile copy gets its block id with v_readlane instead of a scalar load per copy -
    // whose result the copy would have to wait for, together with every LDS read in flight (scalar
    // loads and LDS share one wait counter).
    const int32_t* bt_row = PAGED ? p.block_table + (int64_t)b * p.max_blocks : nullptr;
    int bt_base = k0 >> p.block_shift; // logical block of lane 0 of the first window register
    int32_t bt_win0 = 0, bt_win1 = 0;
    auto bt_fetch = [&](int first) __attribute__((always_inline)) { return bt_row[min(first + lane, p.max_blocks - 1)]; };
    if (PAGED) {
        bt_win0 = bt_fetch(bt_base);
        bt_win1 = bt_fetch(bt_base + 64);
    }
    // moves the window so that it starts at or before logical block `lb_min` (called once per iteration)
    auto bt_advance = [&](int lb_min) __attribute__((always_inline)) {
        if (PAGED && lb_min >= bt_base + 64) { // uniform
            bt_base += 64;
            bt_win0 = bt_win1;
            bt_win1 = bt_fetch(bt_base + 64);
        }
    };
    auto bt_lookup = [&](int lb) __attribute__((always_inline)) {
        const int rel = lb - bt_base; // 0 .. 127 by construction
        int32_t blk = rel < 64 ? __builtin_amdgcn_readlane(bt_win0, rel & 63) : __builtin_amdgcn_readlane(bt_win1, rel & 63);
        if ((uint32_t)blk >= (uint32_t)p.num_blocks) blk = 0; // reported through status
        return blk;
    };
    auto load_tile = [&](auto lfast_tag, auto is_v, int t, u32x4(&r)[BPW]) __attribute__((always_inline)) {
        constexpr bool LFAST = decltype(lfast_tag)::value;
        constexpr bool ISV = decltype(is_v)::value;
        if constexpr (LFAST && PAGED) {
            // a full tile of a paged cache: the RPI rows of a copy block lie in one cache block, so the
            // address is a wave-uniform base (block id from the window, KV head, first row inside the
            // block - all scalar arithmetic) plus the same per-lane constant as for a contiguous cache
#pragma unroll
            for (int j = 0; j < BPW; ++j) {
                const int i = wave * BPW + j; // uniform per wave
                if (NW * BPW == BPS || i < BPS) {
                    const int r0 = k0 + t * kTileKeys + RPI * i;
                    const int64_t sbase = head_base + (int64_t)bt_lookup(r0 >> p.block_shift) * p.stride_block +
                                          (int64_t)((r0 & (p.block_size - 1)) * stride_tok);
                    r[j] = *(const u32x4*)((const char*)((ISV ? vbase : kbase) + sbase) + lane_off);
                }
            }
        } else if constexpr (LFAST) {
#pragma unroll
            for (int j = 0; j < BPW; ++j) {
                const int i = wave * BPW + j; // uniform per wave
                if (NW * BPW == BPS || i < BPS) {
                    const uint32_t off = (uint32_t)((t * kTileKeys + RPI * i) * stride_tok) * 2u;
                    r[j] = *(const u32x4*)((ISV ? vfast : kfast) + off + lane_off);
                }
            }
        } else {
            const uint16_t* gbase = ISV ? vbase : kbase;
            if (k0 + t * kTileKeys >= k1) return; // no such tile: its LDS image is never used
#pragma unroll
            for (int j = 0; j < BPW; ++j) {
                const int i = wave * BPW + j;
                if (i < BPS) {
                    const int r0 = k0 + t * kTileKeys + RPI * i; // RPI divides 16: one cache block in paged mode
                    int tok = min(r0 + lrow, k1 - 1);
                    int64_t base = head_base;
                    if (PAGED) {
                        base += (int64_t)bt_lookup(min(r0, k1 - 1) >> p.block_shift) * p.stride_block;
                        tok &= p.block_size - 1;
                    }
                    const uint32_t off = (uint32_t)(tok * stride_tok + lchunk * 8);
                    r[j] = *(const u32x4*)(gbase + base + off);
                }
            }
        }
    };
    auto stash_tile = [&](auto is_v, uint16_t* slot, const u32x4(&r)[BPW]) __attribute__((always_inline)) {
        constexpr bool ISV = decltype(is_v)::value;
#pragma unroll
        for (int j = 0; j < BPW; ++j) {
            const int i = wave * BPW + j;
            if (NW * BPW == BPS || i < BPS) *(u32x4*)((char*)slot + (ISV ? v_st[j] : k_st[j])) = r[j];
        }
    };
    // Copies are grouped per iteration: group g = K(2g+3), K(2g+4), V(2g+1), V(2g+2) is what
    // iteration g writes to LDS. Its loads are issued in iteration g - 2, so two groups are
    // in flight and alternate between two register sets.
    auto load_group = [&](auto lfast_tag, auto set_tag, int g) __attribute__((always_inline)) {
        constexpr int SET = decltype(set_tag)::value;
        load_tile(lfast_tag, std::false_type{}, 2 * g + 3, stage[SET][0]);
        load_tile(lfast_tag, std::false_type{}, 2 * g + 4, stage[SET][1]);
        load_tile(lfast_tag, std::true_type{}, 2 * g + 1, stage[SET][2]);
        load_tile(lfast_tag, std::true_type{}, 2 * g + 2, stage[SET][3]);
    };
    auto stash_group = [&](auto set_tag, int g) __attribute__((always_inline)) {
        constexpr int SET = decltype(set_tag)::value;
        stash_tile(std::false_type{}, sK[(2 * g + 3) & 3], stage[SET][0]);
        stash_tile(std::false_type{}, sK[(2 * g + 4) & 3], stage[SET][1]);
        stash_tile(std::true_type{}, sV[(2 * g + 1) & 3], stage[SET][2]);
        stash_tile(std::true_type{}, sV[(2 * g + 2) & 3], stage[SET][3]);
    };

    // the rest of the prologue copies: group 0 (set 0)
    load_group(std::false_type{}, std::integral_constant<int, 0>{}, 0);

    uint64_t mask[RPW];
#pragma unroll
    for (int rb = 0; rb < RPW; ++rb)
        mask[rb] = p.tree_keys == 0 ? 0ull : (p.tree_mask ? p.tree_mask[(int64_t)b * p.T + node_of[rb]] : ancestor_mask(sp, node_of[rb]));

    float m2[RPW], lsum[RPW]; // running reference (log2 domain, scaled) and this lane's share of the sum
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
    // K fragment of k-step ks (chunk 2*ks + half of row `col`): k_lane[ks & 1] + ks * 256
    const int k_lane[2] = {(col >> 4) * (DB * 512) + half * 128 + ((col & 15) ^ (4 * half)) * 8,
                           (col >> 4) * (DB * 512) + half * 128 + ((col & 15) ^ (8 + 4 * half)) * 8};
    const int t16 = lane & 15;
    const int v_lane = half * 128 + (t16 >> 2) * 32 + ((lane >> 4) & 1) * 16 + ((t16 >> 1) & 1) * 8 + (t16 & 1) * 4;

    // S^T = K . Q^T for one tile: lane (col, half) gets keys 8*(r/4) + 4*half + r%4 of row `col`
    auto qk = [&](f32x16(&s)[RPW], const uint16_t* kslot) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 a = __builtin_bit_cast(bf16x8, *(const u32x4*)(kslot + k_lane[ks & 1] + ks * 256));
#pragma unroll
            for (int rb = 0; rb < RPW; ++rb) {
                if (ks == 0) {
                    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                    s[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][ks], zero, 0, 0, 0);
                } else {
                    s[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][ks], s[rb], 0, 0, 0);
                }
            }
        }
    };
    // O^T += V^T . P^T: the A operand comes from two transposing reads of 4 keys x 16 channels
    auto pv = [&](const uint16_t* vslot, const bf16x8(&pf)[RPW][2]) __attribute__((always_inline)) {
        const uint16_t* tV = vslot + v_lane;
#pragma unroll
        for (int sl = 0; sl < 2; ++sl)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tV + sl * (DB * 512) + db * 512));
                const s16x4 hi =
                    __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tV + sl * (DB * 512) + db * 512 + 256));
                const bf16x8 a = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                for (int rb = 0; rb < RPW; ++rb)
                    acc[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[rb][sl], acc[rb][db], 0, 0, 0);
            }
    };
    // Online softmax of one tile's scores (vector ALU only): masks, running reference and sum,
    // probabilities as bf16 B operands. Returns the factors the accumulators must be scaled
    // by before this tile's probabilities are applied (1 almost always, see kLazy).
    auto softmax = [&](auto masked_tag, int kt, f32x16(&sc)[RPW], bf16x8(&pf)[RPW][2], float(&alpha)[RPW])
                       __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
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
            // lazy reference: moves only when the tile's maximum exceeds it by more than kLazy
            const float mt = mx * p.scale_log2;
            const float m_new = (mt > m2[rb] + kLazy) ? mt : m2[rb];
            const float m_use = (MASKED && m_new == -INFINITY) ? 0.f : m_new; // no visible key yet
            alpha[rb] = __builtin_amdgcn_exp2f(m2[rb] - m_use);
            m2[rb] = m_new;
            float psum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                s[r] = __builtin_amdgcn_exp2f(fmaf(s[r], p.scale_log2, -m_use)); // exp2(-inf) = 0
                psum += s[r];
            }
            lsum[rb] = lsum[rb] * alpha[rb] + psum;
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
    auto rescale = [&](const float(&alpha)[RPW]) __attribute__((always_inline)) {
        bool need = false;
#pragma unroll
        for (int rb = 0; rb < RPW; ++rb) need |= alpha[rb] != 1.f;
        if (__any(need)) {
#pragma unroll
            for (int rb = 0; rb < RPW; ++rb)
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[rb][db][r] *= alpha[rb];
        }
    };

    // One pipeline step for prefix-only tiles with every neighbour present, written slot
    // by slot so that the instruction stream alternates between the two units: slot (f, rb)
    // holds one MFMA (fragment f: the KS fragments of K for S(next), then the 2*DB
    // fragments of V^T for O += V(prev)^T . P(prev)^T), the LDS read of the fragment two
    // slots ahead, and one share of the softmax of S(cur) -> P(cur) for row block rb. The
    // softmax is cut into 16 groups per row block: 4 of running-maximum work (the last one
    // fixes the reference), 8 of two exponentials each, 4 of bf16 packing.
    // copy_tag >= 0 (a register set): the step also carries the iteration's tile copies, one
    // tile per four slots - the staged tile goes to LDS and its registers are refilled with the
    // tile two groups ahead - so that the LDS writes trickle in between the fragment reads
    // instead of arriving as one 32 KB burst that stalls every wave's reads behind it.
    auto fast_step = [&](auto copy_tag, auto lfast_tag, int g, f32x16(&s_next)[RPW], const uint16_t* kslot,
                         const uint16_t* vslot, const bf16x8(&p_prev)[RPW][2], f32x16(&s_cur)[RPW],
                         bf16x8(&p_cur)[RPW][2], float(&alpha)[RPW]) __attribute__((always_inline)) {
        constexpr int CSET = decltype(copy_tag)::value;
        constexpr int NF = KS + 2 * DB; // fragments = MFMA slots per row block
        constexpr int GPS = 16 / NF;    // softmax groups per slot
        static_assert(16 % NF == 0, "softmax groups must divide evenly over the slots");
        constexpr int PF = 2;
        const uint16_t* tK[2] = {kslot + k_lane[0], kslot + k_lane[1]};
        const uint16_t* tV = vslot + v_lane;
        u32x4 frag[PF + 1];
        // slot order: K and V^T fragments alternate, so that consecutive MFMAs never use the
        // same accumulator (a dependent MFMA issued right behind its predecessor stalls the
        // wave's whole instruction stream until the result is back)
        static_assert(KS == 2 * DB, "as many K fragments as V^T fragments");
        auto load_frag = [&](int f) __attribute__((always_inline)) {
            const int h = f >> 1;
            if ((f & 1) == 0) {
                frag[f % (PF + 1)] = *(const u32x4*)(tK[h & 1] + h * 256);
            } else {
                const int sl = h / DB, db = h % DB;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tV + sl * (DB * 512) + db * 512));
                const s16x4 hi =
                    __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tV + sl * (DB * 512) + db * 512 + 256));
                frag[f % (PF + 1)] = __builtin_bit_cast(u32x4, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            }
        };
        float mx[RPW], nm[RPW], psum[RPW], psum2[RPW];
        u32x4 pw[RPW][2];
        auto softmax_group = [&](int rb, int g) __attribute__((always_inline)) {
            f32x16& sc = s_cur[rb];
            if (g < 4) {
                mx[rb] = g == 0 ? max3(max3(sc[0], sc[1], sc[2]), sc[3], sc[3])
                                : max3(max3(mx[rb], sc[4 * g], sc[4 * g + 1]), sc[4 * g + 2], sc[4 * g + 3]);
                if (g == 3) {
                    const float mt = half_max(mx[rb]) * p.scale_log2;
                    const float m_new = (mt > m2[rb] + kLazy) ? mt : m2[rb]; // finite: prefix keys are always visible
                    alpha[rb] = __builtin_amdgcn_exp2f(m2[rb] - m_new);
                    m2[rb] = m_new;
                    nm[rb] = -m_new;
                    psum[rb] = 0.f;
                    psum2[rb] = 0.f;
                }
            } else if (g < 12) {
#pragma unroll
                for (int e = 2 * (g - 4); e < 2 * (g - 4) + 2; ++e)
                    sc[e] = __builtin_amdgcn_exp2f(fmaf(sc[e], p.scale_log2, nm[rb]));
                // the previous group's pair joins the sum here, one group late, so that the add
                // never waits for an exponential; two running sums keep the adds independent. The
                // empty asm keeps each add in its slot (otherwise all sixteen are sunk behind the
                // step as one dependent chain, out of the MFMAs' shadow).
                if (g > 4) {
                    psum[rb] += sc[2 * (g - 5)];
                    psum2[rb] += sc[2 * (g - 5) + 1];
                    asm volatile("" : "+v"(psum[rb]), "+v"(psum2[rb]));
                }
            } else {
                const int q = g - 12, sl = q >> 1;
                if (g == 12) {
                    psum[rb] += sc[14];
                    psum2[rb] += sc[15];
                }
#pragma unroll
                for (int e = 2 * (q & 1); e < 2 * (q & 1) + 2; ++e) {
                    const f32x2 pr = {sc[8 * sl + 2 * e], sc[8 * sl + 2 * e + 1]};
                    pw[rb][sl][e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
                    asm volatile("" : "+v"(pw[rb][sl][e]));
                }
                if (g == 15) lsum[rb] = lsum[rb] * alpha[rb] + (psum[rb] + psum2[rb]);
            }
        };
#pragma unroll
        for (int f = 0; f < PF; ++f) load_frag(f);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            if (f + PF < NF) load_frag(f + PF);
            const bf16x8 a = __builtin_bit_cast(bf16x8, frag[f % (PF + 1)]);
#pragma unroll
            for (int rb = 0; rb < RPW; ++rb) {
                const int h = f >> 1;
                if (f == 0) {
                    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                    s_next[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][0], zero, 0, 0, 0);
                } else if ((f & 1) == 0) {
                    s_next[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][h], s_next[rb], 0, 0, 0);
                } else {
                    const int sl = h / DB, db = h % DB;
                    acc[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p_prev[rb][sl], acc[rb][db], 0, 0, 0);
                }
#pragma unroll
                for (int sg = f * GPS; sg < (f + 1) * GPS; ++sg) softmax_group(rb, sg);
                if constexpr (CSET >= 0) {
                    if (rb == 0 && f % (NF / 4) == 1) {
                        constexpr int SETC = CSET >= 0 ? CSET : 0;
                        const int part = f / (NF / 4); // 0, 1: K(2g+3), K(2g+4); 2, 3: V(2g+1), V(2g+2)
                        if (part == 0) {
                            stash_tile(std::false_type{}, sK[(2 * g + 3) & 3], stage[SETC][0]);
                            load_tile(lfast_tag, std::false_type{}, 2 * (g + 2) + 3, stage[SETC][0]);
                        } else if (part == 1) {
                            stash_tile(std::false_type{}, sK[(2 * g + 4) & 3], stage[SETC][1]);
                            load_tile(lfast_tag, std::false_type{}, 2 * (g + 2) + 4, stage[SETC][1]);
                        } else if (part == 2) {
                            stash_tile(std::true_type{}, sV[(2 * g + 1) & 3], stage[SETC][2]);
                            load_tile(lfast_tag, std::true_type{}, 2 * (g + 2) + 1, stage[SETC][2]);
                        } else {
                            stash_tile(std::true_type{}, sV[(2 * g + 2) & 3], stage[SETC][3]);
                            load_tile(lfast_tag, std::true_type{}, 2 * (g + 2) + 2, stage[SETC][3]);
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int rb = 0; rb < RPW; ++rb)
#pragma unroll
            for (int sl = 0; sl < 2; ++sl) {
                // the empty asm pins the softmax results to this step: without it the compiler
                // sinks the exponentials past the (rare) rescale branch that follows, out of
                // the shadow of the MFMAs
                asm volatile("" : "+v"(pw[rb][sl]));
                p_cur[rb][sl] = __builtin_bit_cast(bf16x8, pw[rb][sl]);
            }
    };

    // Every load so far (tiles, queries, masks) has landed after this wait. Stating it here,
    // outside any branch, also keeps the compiler from re-waiting for the query registers
    // inside the loop, where such a wait would drain the tile copies in flight.
    __builtin_amdgcn_s_waitcnt(wait_vm(0));
    {
        // the early tiles: rows at or past k1 become zeros
        auto stash_tile_live = [&](auto is_v, uint16_t* slot, const u32x4(&r)[BPW], int t) __attribute__((always_inline)) {
            constexpr bool ISV = decltype(is_v)::value;
#pragma unroll
            for (int j = 0; j < BPW; ++j) {
                const int i = wave * BPW + j;
                if (NW * BPW == BPS || i < BPS) {
                    const bool live = k0 + t * kTileKeys + RPI * i + lrow < k1;
                    const u32x4 zero = {0u, 0u, 0u, 0u};
                    *(u32x4*)((char*)slot + (ISV ? v_st[j] : k_st[j])) = live ? r[j] : zero;
                }
            }
        };
        stash_tile_live(std::false_type{}, sK[0], stage[1][0], 0);
        stash_tile_live(std::false_type{}, sK[1], stage[1][1], 1);
        stash_tile_live(std::false_type{}, sK[2], stage[1][2], 2);
        stash_tile_live(std::true_type{}, sV[0], stage[1][3], 0);
    }
    load_group(std::false_type{}, std::integral_constant<int, 1>{}, 1);
    __syncthreads();

    f32x16 sa[RPW], sb[RPW];  // scores of the iteration's first / second tile
    bf16x8 pa[RPW][2], pb[RPW][2];
#pragma unroll
    for (int rb = 0; rb < RPW; ++rb)
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) pb[rb][sl] = __builtin_bit_cast(bf16x8, u32x4{0u, 0u, 0u, 0u});
    if (wave_active) qk(sa, sK[0]);
    __syncthreads(); // slot 0 of the K ring is rewritten at the end of the first iteration

    // Iteration g handles tiles ta = 2g and tb = 2g + 1. CFAST iterations have every
    // neighbour tile present and only prefix keys; the general form checks and masks.
    auto iteration = [&](auto cfast_tag, auto lfast_tag, auto set_tag, int ta) __attribute__((always_inline)) {
        constexpr bool FAST = decltype(cfast_tag)::value;
        // set_tag: the register set of the copy group that this iteration stashes
        using masked_t = std::integral_constant<bool, !FAST>;
        const int tb = ta + 1;
        const int g = ta >> 1;
        // this iteration requests group g + 2 = tiles 2g + 5 .. 2g + 8
        bt_advance(min(k0 + (2 * g + 5) * kTileKeys, k1 - 1) >> p.block_shift);
        // first tile: S(tb), O(ta - 1) | P(ta)
        if (wave_active) {
            float alpha[RPW];
            if constexpr (FAST) {
                // the very first step applies all-zero probabilities to V(0)
                fast_step(std::integral_constant<int, -1>{}, lfast_tag, g, sb, sK[tb & 3], sV[ta ? (ta - 1) & 3 : 0], pb, sa,
                          pa, alpha);
            } else {
                if (tb < n) qk(sb, sK[tb & 3]);
                if (ta > 0) pv(sV[(ta - 1) & 3], pb);
                softmax(masked_t{}, k0 + ta * kTileKeys, sa, pa, alpha);
            }
            rescale(alpha);
        }
        // In the middle of the iteration: group g (requested one and a half iterations ago) goes
        // to LDS and its registers are refilled with group g + 2. The LDS writes complete under
        // the second tile's work; the barrier at the end publishes them for iteration g + 1.
        // (the fast form spreads the same copies over the slots of its second step, see fast_step;
        // waves without rows have no such step and copy here)
        // (with four waves a tile is two blocks per wave and the interleaved form runs out of registers)
        constexpr bool SPREAD = FAST && BPW == 1;
        if (!SPREAD || !wave_active) {
            stash_group(set_tag, g);
            load_group(lfast_tag, set_tag, g + 2);
        }
        // second tile: S(ta + 2), O(ta) | P(tb)
        if (wave_active) {
            float alpha[RPW];
            if constexpr (FAST) {
                using copy_t = std::conditional_t<SPREAD, decltype(set_tag), std::integral_constant<int, -1>>;
                fast_step(copy_t{}, lfast_tag, g, sa, sK[(ta + 2) & 3], sV[ta & 3], pa, sb, pb, alpha);
                rescale(alpha);
            } else {
                if (ta + 2 < n) qk(sa, sK[(ta + 2) & 3]);
                pv(sV[ta & 3], pa);
                if (tb < n) {
                    softmax(masked_t{}, k0 + tb * kTileKeys, sb, pb, alpha);
                    rescale(alpha);
                }
            }
        }
        __syncthreads();
    };
    using T = std::true_type;
    using F = std::false_type;
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    // tiles that end at or before min(S, k1) hold prefix keys only
    const int n_plain = max(0, min(S, k1) - k0) / kTileKeys;
    const int fast_end = min(n_plain, n - 1) & ~1; // CFAST iterations need tiles ta + 1 (plain) and ta + 2 (present)
    // Iterations come in pairs so that the two register sets alternate at compile time. The
    // forms only ever get more general as ta grows (prefix tiles first, copies near the end
    // of the range last), so three loops in a row cover every case. Iteration ta loads
    // group ta/2 + 2 = tiles up to ta + 8.
    int ta = 0;
    for (; ta + 2 < fast_end && ta + 10 < n_full; ta += 4) {
        iteration(T{}, T{}, S0{}, ta);
        iteration(T{}, T{}, S1{}, ta + 2);
    }
    for (; ta + 2 < fast_end; ta += 4) {
        iteration(T{}, F{}, S0{}, ta);
        iteration(T{}, F{}, S1{}, ta + 2);
    }
    for (; ta < n; ta += 4) {
        iteration(F{}, F{}, S0{}, ta);
        if (ta + 2 < n) iteration(F{}, F{}, S1{}, ta + 2);
    }
    if (!wave_active) return;
    if ((n & 1) == 0) pv(sV[(n - 1) & 3], pb);

    // ---- epilogue: lane (col, half) holds, for row `col`, channels db*32 + 8*(r/4) + 4*half + r%4
#pragma unroll
    for (int rb = 0; rb < RPW; ++rb) {
        const int r_local = row_base + rb * kRowBlock + col;
        const float l = half_sum(lsum[rb]);
        if (whole) {
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
            const int64_t unit = BAL ? kvh : (int64_t)b * p.Hkv + kvh;
            const int64_t blk = part_block(p, unit, slot, (row_base >> 5) + rb);
            uint16_t* po = p.part_o + blk * (kRowBlock * D);
            const float inv = l > 0.f ? 1.f / l : 0.f; // no visible key in this split: zeros, weight 0
#pragma unroll
            for (int db = 0; db < DB; ++db) store_partial<D>(po, db, lane, acc[rb][db], inv);
            if (half == 0) {
                const f32x2 ml = {m2[rb], l};
                const int64_t mlb = ml_block(p, unit, slot, (row_base >> 5) + rb);
                *(f32x2*)(p.part_ml + (mlb + col) * 2) = ml;
            }
        }
    }
    }; // run_piece

    if constexpr (!BAL) {
        // workgroup id -> (sequence, KV head, row group, split), XCD-aware (see attention_mfma.hip)
        const int per_xcd = (p.total_wgs + 7) >> 3;
        const int v = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
        if (v >= p.total_wgs) return;
        const int split = v % p.num_splits; // splits fastest, see attention_mfma.hip
        int rest = v / p.num_splits;
        const int rg = rest % p.row_groups;
        rest /= p.row_groups;
        const int kvh = rest % p.Hkv;
        const int b = rest / p.Hkv;
        // the host keeps every split's first key below max_prefix_len + tree_keys, hence inside the cache
        run_piece(b, kvh, rg, split * p.keys_per_split, p.keys_per_split, split, p.num_splits == 1);
    } else {
        // workgroup id -> (share, KV head, row group): the row groups of a (share, KV head) sit next to each
        // other on one XCD (they read the same keys), consecutive (share, KV head) pairs on different ones
        const int xj = blockIdx.x >> 3;
        const int rg = xj % p.row_groups;
        const int u = (xj / p.row_groups) * 8 + (blockIdx.x & 7);
        const int c = u / p.Hkv, kvh = u % p.Hkv;
        if (c >= p.bal_chunks) return;
        int start, steps, total;
        bool usable;
        bal_scan(p, lane, start, steps, total, usable);
        // sequences that no piece will ever visit report their bad prefix length here
        if (c == 0 && kvh == 0 && rg == 0 && wave == 0 && lane < p.B && !usable && p.status) p.status[lane] = VS_STATUS_BAD_PREFIX;
        const int bounds = bal_bounds(p, lane, start, steps, total);
        if (c == 0 && kvh == 0 && rg == 0 && wave == 0) p.bal_table[lane] = bounds; // for the combine kernel
        const int lo = __builtin_amdgcn_readlane(bounds, c);
        const int hi = c + 1 < p.bal_chunks ? __builtin_amdgcn_readlane(bounds, c + 1) : total;
        for (int i = 0; i < p.B; ++i) {
            const int s0 = __builtin_amdgcn_readlane(start, i), t = __builtin_amdgcn_readlane(steps, i);
            int t0, t1;
            if (bal_piece(lo, hi, s0, t, t0, t1)) { // uniform
                __syncthreads(); // the previous piece's last reads of the tile rings, the tree and the flag
                run_piece(i, kvh, rg, t0 * kIterKeys, (t1 - t0) * kIterKeys, c + i, t0 == 0 && t1 == t);
            }
        }
    }
}

template <int D, int RPW, int NW>
hipError_t launch_pipe(const AttnParams& p, hipStream_t s) {
    if (p.bal_chunks > 0) {
        const dim3 grid(((p.bal_chunks * p.Hkv + 7) / 8) * 8 * p.row_groups);
        if (p.paged) hipLaunchKernelGGL((attn_mfma_pipe_kernel<D, RPW, NW, true, true>), grid, dim3(NW * kWave), 0, s, p);
        else hipLaunchKernelGGL((attn_mfma_pipe_kernel<D, RPW, NW, false, true>), grid, dim3(NW * kWave), 0, s, p);
        return hipGetLastError();
    }
    const dim3 grid(((p.total_wgs + 7) / 8) * 8);
    if (p.paged) hipLaunchKernelGGL((attn_mfma_pipe_kernel<D, RPW, NW, true, false>), grid, dim3(NW * kWave), 0, s, p);
    else hipLaunchKernelGGL((attn_mfma_pipe_kernel<D, RPW, NW, false, false>), grid, dim3(NW * kWave), 0, s, p);
    return hipGetLastError();
}

} // namespace

// One row block per wave; four waves (two workgroups per CU) or eight.
bool attention_pipe_supported(int rpw, int waves) { return rpw == 1 && (waves == 4 || waves == 8); }

hipError_t launch_attention_mfma_pipe(const AttnParams& p, int rpw, int waves, hipStream_t s) {
    if (!attention_pipe_supported(rpw, waves) || (p.d != 128 && p.d != 64)) return hipErrorInvalidValue;
    if (p.d == 128) return waves == 8 ? launch_pipe<128, 1, 8>(p, s) : launch_pipe<128, 1, 4>(p, s);
    return waves == 8 ? launch_pipe<64, 1, 8>(p, s) : launch_pipe<64, 1, 4>(p, s);
}

} // namespace vs
