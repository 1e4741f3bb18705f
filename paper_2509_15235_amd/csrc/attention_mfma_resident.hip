// Tree-masked attention for small launches (one layer of one sequence): the whole key range
// of a split is resident in LDS and the keys are split once more inside the workgroup.
//
// Math and MFMA layouts are those of attention_mfma.hip (paper Eq. 1 with a softmax scale over
// the prefix plus the ancestor-or-self tree slots, Section 3.1): S^T = K . Q^T with
// v_mfma_f32_32x32x16_bf16, a lane holds 16 keys of ONE query row, the probabilities are the
// B operand of O^T += V^T . P^T, V is transposed by ds_read_b64_tr_b16 on its way out of LDS.
//
// Why another schedule. A launch with few (sequence, KV head) units is latency-bound: with one
// wave per SIMD the streaming kernel spends 2 us per 64-key iteration of which the matrix cores
// work 0.4 us - the rest is a single wave issuing its tile copy, LDS writes, barrier and
// softmax one dependent instruction after the other. Here a workgroup of eight waves owns
// NRB row blocks x KQ = 8 / NRB key parts of a split of NT 32-key tiles (at most 192 keys,
// 96 KB). Every load of the split is issued at once, before anything is waited for, ordered by
// stage: stage j holds the j-th tile of every key part. As soon as a stage has arrived it goes
// into LDS (one barrier) and every wave runs that tile for its row block while the later stages
// are still on their way (wall-clock stamps of the earlier form - all loads, one barrier, then
// all tiles - showed 3.4 us until the data was there, 1.5 us to put it into LDS and 2.2 - 3.4 us
// of tiles, one after the other). Tiles never share an LDS slot, so one barrier per stage is all
// the synchronisation there is; two waves per SIMD cover each other's stalls; the key parts are
// merged through LDS (log-sum-exp, like the combine kernel does for the splits). Split partials
// and final rows leave as in the streaming kernels, so the combine kernel and the workspace
// layout are shared.
#include <type_traits>

#include "attn_mfma_common.h"

namespace vs {

namespace {

constexpr int kResWaves = 8;
constexpr int kResMaxTiles = kResidentMaxKeys / kTileKeys; // 32-key tiles of one split

template <int D, int NRB, int NT>
__global__ __launch_bounds__(kResWaves * 64, 2) void attn_mfma_resident_kernel(const AttnParams p) {
    constexpr int KS = D / 16;          // k-steps of the S^T product
    constexpr int DB = D / 32;          // 32-channel blocks of the output
    constexpr int KQ = kResWaves / NRB; // key parts inside the workgroup
    constexpr int PPM = (NT + KQ - 1) / KQ; // tiles per key part = stages
    constexpr int SUB = kTileKeys * D;  // elements per 32-key tile of K (or V)
    constexpr int BPS = SUB * 2 / 1024; // 1 KB copy blocks per tile
    constexpr int LPR = D / 8;          // lanes (16-byte chunks) per row
    constexpr int RPI = 64 / LPR;       // rows per load instruction
    constexpr int SPW = (KQ * BPS + kResWaves - 1) / kResWaves; // copy blocks per wave, stage and tensor
    constexpr int TILE_BYTES = 2 * NT * SUB * 2;
    constexpr int MERGE_BYTES = kResWaves * (DB * 1024 + 128) * 4; // every wave's exchange area: accumulators, max, sum
    constexpr int SMEM_ELEMS = (TILE_BYTES > MERGE_BYTES ? TILE_BYTES : MERGE_BYTES) / 2;
    static_assert(NT >= 1 && NT <= kResMaxTiles, "a split holds at most kResidentMaxKeys keys");

    // tiles: K[t] at smem + t*SUB, V[t] at smem + (NT + t)*SUB; after the last tile has been
    // consumed the same memory carries the key parts' results to the merging waves
    __shared__ __attribute__((aligned(1024))) uint16_t smem[SMEM_ELEMS];
    __shared__ int32_t sp[VS_MAX_TREE];
    __shared__ int32_t sflag;
    uint16_t* sK = smem;
    uint16_t* sV = smem + NT * SUB;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5;
    const int col = lane & 31;
    const int rbw = wave % NRB; // row block inside the group
    const int kq = wave / NRB;  // key part

    // workgroup id -> (sequence, KV head, row group, split); same XCD-aware remap as the other kernels
    const int per_xcd = (p.total_wgs + 7) >> 3;
    const int v = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (v >= p.total_wgs) return;
    // splits fastest: all key splits of a (sequence, KV head, row group) run on one XCD, the one
    // that the combine workgroups of those rows are placed on by the same remap (see attention_mfma.hip)
    const int split = v % p.num_splits;
    int rest = v / p.num_splits;
    const int rg = rest % p.row_groups;
    rest /= p.row_groups;
    const int kvh = rest % p.Hkv;
    const int b = rest / p.Hkv;

    const int32_t S = p.prefix_len[b]; // requested first, needed last: everything below is issued before it arrives

    // ---- copy the split's keys and values. Stage j = tile j of every key part (tile kq * PPM + j);
    // inside a stage, copy block i = (key part i / BPS, rows RPI * (i % BPS) ..) and wave w takes
    // blocks w, w + 8, ...; one load instruction reads RPI whole rows (1 KB of consecutive memory).
    // The loads do not wait for the prefix length: they are clamped to the cache (not to the
    // sequence), and rows that turn out to lie past the sequence's last key are zeroed on their
    // way into LDS (whatever the cache holds there - NaN included - must not meet a zero
    // probability in the V product). A block-table entry outside the pool reads block 0. Chunk c
    // of tile row r lands where the fragment reads expect it (same placement as the streaming
    // kernel):
    //   K: ((r/16)*DB + c/4) * 1024 + (c%4) * 256 + ((r%16) ^ 4*(c%4)) * 16
    //   V: ((r/16)*DB + c/4) * 1024 + (4*(r%16) + c%4) * 16
    // (No branch around a block's loads or stores: a conditional assignment of the staging
    // array makes the compiler spill the whole array at every branch. Slots of tiles past the
    // split's last one receive zeros and are never read.)
    const uint16_t* kbase = (const uint16_t*)p.k;
    const uint16_t* vbase = (const uint16_t*)p.v;
    const int64_t head_base = (p.paged ? 0 : (int64_t)b * p.stride_seq) + (int64_t)kvh * p.stride_head;
    const int stride_tok = (int)p.stride_tok;
    const int lrow = lane / LPR, lchunk = lane % LPR;
    const int k0 = split * p.keys_per_split; // the host keeps k0 below max_prefix_len + tree_keys, hence inside the cache
    const int64_t cache_tokens = p.paged ? (int64_t)p.max_blocks * p.block_size : p.capacity;
    const int kend = (int)(cache_tokens < (int64_t)k0 + p.keys_per_split ? cache_tokens : (int64_t)k0 + p.keys_per_split);
    u32x4 kreg[PPM][SPW], vreg[PPM][SPW];
    // tile and first row (inside the tile) of this wave's u-th copy block of stage j; blocks past the
    // stage's last one (KQ * BPS not a multiple of the wave count) repeat its last block
    auto block_tile = [&](int j, int u) __attribute__((always_inline)) {
        const int i = min(wave + kResWaves * u, KQ * BPS - 1);
        return min((i / BPS) * PPM + j, NT - 1);
    };
    auto block_row = [&](int u) __attribute__((always_inline)) {
        const int i = min(wave + kResWaves * u, KQ * BPS - 1);
        return (i % BPS) * RPI;
    };
    auto issue_stage = [&](auto is_v, int j) __attribute__((always_inline)) {
        constexpr bool ISV = decltype(is_v)::value;
#pragma unroll
        for (int u = 0; u < SPW; ++u) {
            const int r0 = min(k0 + kTileKeys * block_tile(j, u) + block_row(u), kend - 1); // RPI divides 16: one cache block in paged mode
            int tok = min(r0 + lrow, kend - 1);
            int64_t base = head_base;
            if (p.paged) {
                int32_t blk = p.block_table[(int64_t)b * p.max_blocks + (r0 >> p.block_shift)];
                if ((uint32_t)blk >= (uint32_t)p.num_blocks) blk = 0; // reported through status
                base += (int64_t)blk * p.stride_block;
                tok &= p.block_size - 1;
            }
            const uint32_t off = (uint32_t)(tok * stride_tok + lchunk * 8);
            if constexpr (ISV) vreg[j][u] = *(const u32x4*)(vbase + base + off);
            else kreg[j][u] = *(const u32x4*)(kbase + base + off);
        }
    };
    issue_stage(std::false_type{}, 0); // the first keys lead: the first scores need them and the queries

    // ---- this wave's rows, mask and queries (in flight together with the tiles)
    const int row_base = rg * (NRB * kRowBlock) + rbw * kRowBlock;
    const bool wave_active = row_base < p.rows;
    const int r = min(row_base + col, p.rows - 1); // rows past the end repeat the last row (results discarded)
    const int node = r / p.group;
    const int hq = kvh * p.group + (r - node * p.group);
    bf16x8 qf[KS];
    {
        const uint16_t* qr = (const uint16_t*)p.q + (((int64_t)b * p.T + node) * p.Hq + hq) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qr + ks * 16));
    }
    // the row's ancestor mask, when the caller supplies the masks: requested ahead of the later stages
    uint64_t mask_given = 0;
    if (p.tree_mask && p.tree_keys != 0) mask_given = p.tree_mask[(int64_t)b * p.T + node];
    issue_stage(std::true_type{}, 0);
#pragma unroll
    for (int j = 1; j < PPM; ++j) {
        issue_stage(std::false_type{}, j);
        issue_stage(std::true_type{}, j);
    }

    int32_t tree_code = VS_STATUS_OK;
    if (p.tree_mask || p.tree_keys == 0) {
        if (tid == 0) sflag = 0;
        __syncthreads();
    } else {
        tree_code = load_tree(p.parent + (int64_t)b * p.T, p.T, sp, &sflag);
    }
    const uint64_t mask = p.tree_keys == 0 ? 0ull : (p.tree_mask ? mask_given : (tree_code == VS_STATUS_OK ? ancestor_mask(sp, node) : 0ull));
    const bool s_ok = prefix_ok(p, S);
    if (kvh == 0 && split == 0 && rg == 0) report_status(p, b, tree_code, s_ok, S, &sflag);
    if (tree_code != VS_STATUS_OK || !s_ok) return;

    const int nk = S + p.tree_keys;
    if (k0 >= nk) return;
    const int k1 = min(nk, k0 + p.keys_per_split);
    const int nt = (k1 - k0 + kTileKeys - 1) / kTileKeys; // tiles of this split, <= kResMaxTiles

    // ---- this wave's key part: tiles kq * PPM + j, j = 0 .. PPM - 1 (those below nt)
    float m2 = -INFINITY, lsum = 0.f; // running reference (log2 domain, scaled) and this lane's share of the sum
    f32x16 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[db][q] = 0.f;

    // per-lane LDS offsets (elements); everything else is a compile-time immediate
    const int k_lane[2] = {(col >> 4) * (DB * 512) + half * 128 + ((col & 15) ^ (4 * half)) * 8,
                           (col >> 4) * (DB * 512) + half * 128 + ((col & 15) ^ (8 + 4 * half)) * 8};
    const int t16 = lane & 15;
    const int v_lane = half * 128 + (t16 >> 2) * 32 + ((lane >> 4) & 1) * 16 + ((t16 >> 1) & 1) * 8 + (t16 & 1) * 4;

    auto tile = [&](auto masked_tag, int t) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        const uint16_t* kt_ = sK + t * SUB;
        const uint16_t* vt_ = sV + t * SUB + v_lane;
        // S^T = K . Q^T: lane (col, half) gets keys 8*(q/4) + 4*half + q%4 of row `col`
        f32x16 s;
#pragma unroll
        for (int q = 0; q < 16; ++q) s[q] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 a = __builtin_bit_cast(bf16x8, *(const u32x4*)(kt_ + k_lane[ks & 1] + ks * 256));
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s, 0, 0, 0);
        }
        if constexpr (MASKED) {
            const int rel = k0 + t * kTileKeys + 4 * half - S; // tree slot of this lane's key 0 (negative: prefix)
            const uint32_t tree_end = (uint32_t)(k1 - S);
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int sh = rel + 8 * (q >> 2) + (q & 3);
                const uint32_t bit = (uint32_t)(mask >> (sh & 63)) & 1u;
                const bool vis = (sh < 0) | (((uint32_t)sh < tree_end) & (bit != 0));
                s[q] = vis ? s[q] : -INFINITY;
            }
        }
        float mx = max3(s[0], s[1], s[2]);
#pragma unroll
        for (int q = 3; q < 15; q += 2) mx = max3(mx, s[q], s[q + 1]);
        mx = fmaxf(mx, s[15]);
        mx = half_max(mx);
        // lazy reference: moves only when the tile's maximum exceeds it by more than kLazy
        const float mt = mx * p.scale_log2;
        const float m_new = (mt > m2 + kLazy) ? mt : m2;
        const float m_use = (MASKED && m_new == -INFINITY) ? 0.f : m_new; // no visible key yet
        const float alpha = __builtin_amdgcn_exp2f(m2 - m_use);
        m2 = m_new;
        float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
        for (int q = 0; q < 16; q += 2) {
            s[q] = __builtin_amdgcn_exp2f(fmaf(s[q], p.scale_log2, -m_use)); // exp2(-inf) = 0
            s[q + 1] = __builtin_amdgcn_exp2f(fmaf(s[q + 1], p.scale_log2, -m_use));
            ps0 += s[q];
            ps1 += s[q + 1];
        }
        lsum = lsum * alpha + (ps0 + ps1);
        if (__any(alpha != 1.f)) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[db][q] *= alpha;
        }
        bf16x8 pf[2];
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) {
            u32x4 w;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const f32x2 pr = {s[8 * sl + 2 * e], s[8 * sl + 2 * e + 1]};
                w[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
            }
            pf[sl] = __builtin_bit_cast(bf16x8, w);
        }
        // O^T += V^T . P^T: the A operand comes from two transposing reads of 4 keys x 16 channels
#pragma unroll
        for (int sl = 0; sl < 2; ++sl)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vt_ + sl * (DB * 512) + db * 512));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vt_ + sl * (DB * 512) + db * 512 + 256));
                const bf16x8 a = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[sl], acc[db], 0, 0, 0);
            }
    };
    // tiles that end at or before min(S, k1) hold prefix keys only
    const int n_plain = max(0, min(S, k1) - k0) / kTileKeys;
#pragma unroll
    for (int j = 0; j < PPM; ++j) {
        // stage j has arrived once at most the later stages' loads are outstanding (loads return in
        // order; the compiler counts them and waits for exactly that before the first use below)
#pragma unroll
        for (int u = 0; u < SPW; ++u) {
            if (SPW * kResWaves == KQ * BPS || wave + kResWaves * u < KQ * BPS) { // uniform per wave
                const int t = block_tile(j, u), rr = block_row(u) + lrow, c = lchunk;
                const bool live = k0 + kTileKeys * t + rr < k1;
                const u32x4 zero = {0u, 0u, 0u, 0u};
                const uint32_t ko = (uint32_t)(((rr >> 4) * DB + (c >> 2)) * 1024 + (c & 3) * 256 + (((rr & 15) ^ (4 * (c & 3))) * 16));
                const uint32_t vo = (uint32_t)(((rr >> 4) * DB + (c >> 2)) * 1024 + (4 * (rr & 15) + (c & 3)) * 16);
                *(u32x4*)((char*)(sK + t * SUB) + ko) = live ? kreg[j][u] : zero;
                *(u32x4*)((char*)(sV + t * SUB) + vo) = live ? vreg[j][u] : zero;
            }
        }
        __syncthreads();
        const int t = kq * PPM + j;
        if (wave_active && t < nt) {
            if (t < n_plain) tile(std::false_type{}, t);
            else tile(std::true_type{}, t);
        }
    }

    // ---- merge the key parts through LDS (log-sum-exp) and write the rows. The work is shared: a row
    // block's accumulators are 2 * DB pieces of eight registers (piece = channel block * 2 + half of
    // its registers, the 16-byte unit of the partial-result layout); key part k owns pieces
    // k * PPK .. (k + 1) * PPK - 1, receives the other parts' versions of those, merges them in ascending
    // part order (so every wave of a row block computes the same sum) and stores them. Every wave
    // hands (8 - PPK pieces, max, sum) over and takes as much back, instead of part 0 doing all of it.
    __syncthreads(); // every wave is done with the tiles
    float* sm = (float*)smem;
    constexpr int NP = 2 * DB;                    // pieces per row block
    constexpr int PPK = NP / KQ > 0 ? NP / KQ : 1; // pieces owned by a key part
    constexpr int OWNERS = NP / PPK;              // key parts that own pieces (all of them unless KQ > NP)
    constexpr int XCH = NP * 512 + 128;           // floats a wave's exchange area holds: pieces [piece][2][64 lanes][4], max[64], sum[64]
    static_assert(kResWaves * XCH * 4 <= SMEM_ELEMS * 2, "exchange area fits");
    float* mine = sm + (rbw * KQ + kq) * XCH;
    auto piece_owner = [](int pc) { return pc / PPK; };
    if (wave_active) {
#pragma unroll
        for (int pc = 0; pc < NP; ++pc) {
            // written by everybody but the owner; which pieces those are depends on kq, the registers
            // they come from do not
            if (piece_owner(pc) != kq) {
                const int db = pc >> 1, hp = pc & 1;
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    const f32x4 w = {acc[db][8 * hp + 4 * hh], acc[db][8 * hp + 4 * hh + 1], acc[db][8 * hp + 4 * hh + 2],
                                     acc[db][8 * hp + 4 * hh + 3]};
                    *(f32x4*)(mine + pc * 512 + hh * 256 + lane * 4) = w;
                }
            }
        }
        mine[NP * 512 + lane] = m2;
        mine[NP * 512 + 64 + lane] = lsum;
    }
    __syncthreads();
    if (!wave_active || kq >= OWNERS) return;

    // reference and sum over all key parts, the same arithmetic in every wave of the row block
    float mo[KQ], lo[KQ];
#pragma unroll
    for (int o = 0; o < KQ; ++o) {
        const float* src = sm + (rbw * KQ + o) * XCH;
        mo[o] = src[NP * 512 + lane];
        lo[o] = src[NP * 512 + 64 + lane];
    }
    float M = mo[0];
#pragma unroll
    for (int o = 1; o < KQ; ++o) M = fmaxf(M, mo[o]);
    const float Ms = (M == -INFINITY) ? 0.f : M; // no part has seen a visible key: every factor below is 2^-inf = 0
    float fo[KQ], lall = 0.f;
#pragma unroll
    for (int o = 0; o < KQ; ++o) {
        fo[o] = __builtin_amdgcn_exp2f(mo[o] - Ms);
        lall += lo[o] * fo[o];
    }
    const float l = half_sum(lall);
    const int r_local = row_base + col;
    const bool final_rows = p.num_splits == 1;
    const float inv = final_rows ? 1.f / l : (l > 0.f ? 1.f / l : 0.f); // partials: no visible key in this split -> zeros, weight 0
    uint16_t* orow = (uint16_t*)p.out + (((int64_t)b * p.T + node) * p.Hq + hq) * D;
    uint16_t* po = p.part_o + part_block(p, (int64_t)b * p.Hkv + kvh, split, row_base >> 5) * (kRowBlock * D);

    // this wave's pieces: lane (col, half) holds, for row `col`, channels db*32 + 8*(q/4) + 4*half + q%4
    auto finish = [&](auto kq_tag) __attribute__((always_inline)) {
        constexpr int MY = decltype(kq_tag)::value;
#pragma unroll
        for (int i = 0; i < PPK; ++i) {
            const int pc = MY * PPK + i, db = pc >> 1, hp = pc & 1;
            float r[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) r[e] = 0.f;
#pragma unroll
            for (int o = 0; o < KQ; ++o) {
                if (o == MY) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) r[e] += fo[o] * acc[db][8 * hp + e];
                } else {
                    const float* src = sm + (rbw * KQ + o) * XCH + pc * 512 + lane * 4;
                    const f32x4 a0 = *(const f32x4*)src, a1 = *(const f32x4*)(src + 256);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        r[e] += fo[o] * a0[e];
                        r[4 + e] += fo[o] * a1[e];
                    }
                }
            }
            if (final_rows) {
                if (r_local < p.rows) {
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        u32x2 w;
                        w[0] = pack_bf16x2(r[4 * hh] * inv, r[4 * hh + 1] * inv);
                        w[1] = pack_bf16x2(r[4 * hh + 2] * inv, r[4 * hh + 3] * inv);
                        *(u32x2*)(orow + db * 32 + 8 * (2 * hp + hh) + 4 * half) = w;
                    }
                }
            } else {
                const u32x2 w0 = pack_partial(r[0], r[1], r[2], r[3], inv), w1 = pack_partial(r[4], r[5], r[6], r[7], inv);
                const u32x4 w = {w0[0], w0[1], w1[0], w1[1]};
                *(u32x4*)(po + (pc * 64 + lane) * 8) = w;
            }
        }
    };
    switch (kq) { // uniform per wave; the case fixes which registers are this wave's
    case 0: finish(std::integral_constant<int, 0>{}); break;
    case 1: finish(std::integral_constant<int, 1 % OWNERS>{}); break;
    case 2: finish(std::integral_constant<int, 2 % OWNERS>{}); break;
    case 3: finish(std::integral_constant<int, 3 % OWNERS>{}); break;
    case 4: finish(std::integral_constant<int, 4 % OWNERS>{}); break;
    case 5: finish(std::integral_constant<int, 5 % OWNERS>{}); break;
    case 6: finish(std::integral_constant<int, 6 % OWNERS>{}); break;
    default: finish(std::integral_constant<int, 7 % OWNERS>{}); break;
    }
    if (!final_rows && kq == 0 && half == 0) {
        const f32x2 ml = {M, l};
        const int64_t mlb = ml_block(p, (int64_t)b * p.Hkv + kvh, split, row_base >> 5);
        *(f32x2*)(p.part_ml + (mlb + col) * 2) = ml;
    }
}

template <int D, int NRB, int NT>
hipError_t launch_res(const AttnParams& p, hipStream_t s) {
    const dim3 grid(((p.total_wgs + 7) / 8) * 8);
    hipLaunchKernelGGL((attn_mfma_resident_kernel<D, NRB, NT>), grid, dim3(kResWaves * kWave), 0, s, p);
    return hipGetLastError();
}

// NT = tiles per split (2, 4 or 6 tiles of 32 keys)
template <int D, int NRB>
hipError_t launch_res_nt(const AttnParams& p, hipStream_t s) {
    const int nt = p.keys_per_split / kTileKeys;
    if (nt <= 2) return launch_res<D, NRB, 2>(p, s);
    if (nt <= 4) return launch_res<D, NRB, 4>(p, s);
    return launch_res<D, NRB, 6>(p, s);
}

} // namespace

// Row blocks per workgroup: 4, 2 or 1 (the other waves split the keys).
bool attention_resident_supported(int row_blocks) { return row_blocks == 4 || row_blocks == 2 || row_blocks == 1; }

hipError_t launch_attention_mfma_resident(const AttnParams& p, int row_blocks, hipStream_t s) {
    if (!attention_resident_supported(row_blocks) || p.keys_per_split > kResidentMaxKeys || p.keys_per_split % kIterKeys) return hipErrorInvalidValue;
    if (p.d == 128) {
        return row_blocks == 4 ? launch_res_nt<128, 4>(p, s) : (row_blocks == 2 ? launch_res_nt<128, 2>(p, s) : launch_res_nt<128, 1>(p, s));
    }
    if (p.d == 64) {
        return row_blocks == 4 ? launch_res_nt<64, 4>(p, s) : (row_blocks == 2 ? launch_res_nt<64, 2>(p, s) : launch_res_nt<64, 1>(p, s));
    }
    return hipErrorInvalidValue;
}

} // namespace vs
