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
// accumulators in registers for the whole key range. Keys stream through LDS in tiles
// of 32: K as stored ([key][d]), V transposed ([d][key]).
//
// Per tile and row block (v_mfma_f32_32x32x16_bf16, A = 32x16, B = 16x32, C = 32x32):
//   S^T[key][row] = K[key][:] . Q[row][:]        A = K tile (LDS), B = Q (registers)
//   online softmax along keys: a lane holds 16 keys of ONE row, so the row's ancestor
//   mask, running max and running sum are plain per-lane scalars
//   O^T[d][row] += V^T[d][key] . P^T[key][row]   A = V^T tile (LDS), B = P (registers:
//   the C layout of S^T is, after rounding to bf16, already a B operand; V^T is stored
//   in LDS with the matching key order)
//
// With one split the normalised result is written as bf16; otherwise unnormalised
// partials (O, running max, running sum) go to the workspace for the combine kernel.
#include "vs_device.h"

namespace vs {

namespace {

constexpr int kKPad = 8; // bf16 elements of padding per LDS row (keeps 16-byte reads conflict-free)

// Position of tile-local key `key` (0..31) inside a V^T row. The MFMA C layout gives
// lane half h of a 32x32 block keys {8a + 4h + c}; as a B operand that lane must hold 8
// consecutive contraction indices, so keys are stored with bits a (8s) and h (4s) swapped.
__device__ __forceinline__ int vt_pos(int key) {
    return (key & 16) | ((key & 4) << 1) | ((key & 8) >> 1) | (key & 3);
}

template <int D, int RPW, int NW>
__global__ __launch_bounds__(NW * 64) void attn_mfma_kernel(const AttnParams p) {
    constexpr int NT = NW * kWave;
    constexpr int KS = D / 16;              // k-steps of the S^T product
    constexpr int DB = D / 32;              // 32-channel blocks of the output
    constexpr int CPR = D / 8;              // 16-byte chunks per key row
    constexpr int CHUNKS = kTileKeys * CPR; // chunks per K (or V) tile
    constexpr int CPT = (CHUNKS + NT - 1) / NT;

    __shared__ __attribute__((aligned(16))) uint16_t sK[kTileKeys][D + kKPad];
    __shared__ __attribute__((aligned(16))) uint16_t sVt[D][kTileKeys + kKPad];
    __shared__ int32_t sp[VS_MAX_TREE];
    __shared__ int32_t sflag;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int half = lane >> 5;
    const int col = lane & 31;

    // Workgroup id -> (sequence, KV head, split, row group). Consecutive hardware ids go
    // round-robin over the 8 XCDs; the remap keeps workgroups that read the same K/V
    // (row groups, then neighbouring splits) on one XCD so they share its L2.
    const int per_xcd = (p.total_wgs + 7) >> 3;
    const int v = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (v >= p.total_wgs) return;
    const int rg = v % p.row_groups;
    int rest = v / p.row_groups;
    const int split = rest % p.num_splits;
    rest /= p.num_splits;
    const int kvh = rest % p.Hkv;
    const int b = rest / p.Hkv;

    const int32_t tree_code = load_tree(p.parent + (int64_t)b * p.T, p.T, sp, &sflag);
    const int32_t S = p.prefix_len[b];
    const bool s_ok = prefix_ok(p, S);
    if (kvh == 0 && split == 0 && rg == 0) report_status(p, b, tree_code, s_ok, S, &sflag);
    if (tree_code != VS_STATUS_OK || !s_ok) return;

    const int nk = S + p.T;
    const int k0 = split * p.keys_per_split;
    if (k0 >= nk) return;
    const int k1 = min(nk, k0 + p.keys_per_split);

    // ---- this wave's rows, their masks and queries
    const int row_base = rg * p.rows_per_group + wave * (RPW * kRowBlock);
    const bool wave_active = row_base < p.rows;
    uint64_t mask[RPW];
    bf16x8 qf[RPW][KS];
    const uint16_t* qbase = (const uint16_t*)p.q;
#pragma unroll
    for (int rb = 0; rb < RPW; ++rb) {
        const int r = row_base + rb * kRowBlock + col;
        mask[rb] = 0;
        if (r < p.rows) {
            const int node = r / p.group;
            const int hq = kvh * p.group + (r - node * p.group);
            mask[rb] = p.tree_mask ? p.tree_mask[(int64_t)b * p.T + node] : ancestor_mask(sp, node);
            const uint16_t* qr = qbase + (((int64_t)b * p.T + node) * p.Hq + hq) * D + half * 8;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                qf[rb][ks] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qr + ks * 16));
        } else {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) qf[rb][ks] = __builtin_bit_cast(bf16x8, u32x4{0, 0, 0, 0});
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

    const uint16_t* kbase = (const uint16_t*)p.k;
    const uint16_t* vbase = (const uint16_t*)p.v;
    u32x4 kreg[CPT], vreg[CPT];

    auto fetch = [&](int kt) {
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int c = tid + i * NT;
            kreg[i] = u32x4{0, 0, 0, 0};
            vreg[i] = u32x4{0, 0, 0, 0};
            if (c < CHUNKS) {
                const int key = c / CPR, dc = c % CPR;
                const int tok = kt + key;
                if (tok < k1) { // slots past the last valid token stay zero in LDS
                    const int64_t off = token_offset(p, b, kvh, tok) + dc * 8;
                    kreg[i] = *(const u32x4*)(kbase + off);
                    vreg[i] = *(const u32x4*)(vbase + off);
                }
            }
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int c = tid + i * NT;
            if (c < CHUNKS) {
                const int key = c / CPR, dc = c % CPR;
                *(u32x4*)&sK[key][dc * 8] = kreg[i];
                const int pos = vt_pos(key);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    sVt[dc * 8 + 2 * e][pos] = (uint16_t)(vreg[i][e] & 0xffffu);
                    sVt[dc * 8 + 2 * e + 1][pos] = (uint16_t)(vreg[i][e] >> 16);
                }
            }
        }
    };

    fetch(k0);
    for (int kt = k0; kt < k1; kt += kTileKeys) {
        __syncthreads(); // previous tile fully consumed
        stash();
        __syncthreads();
        if (kt + kTileKeys < k1) fetch(kt + kTileKeys); // in flight while this tile is computed
        if (!wave_active) continue;

        // ---- per row block: S^T = K . Q^T, mask, online softmax, P as a B operand.
        // Lane (col, half) holds keys 8*(r/4) + 4*half + r%4 of row `col`.
        const bool need_mask = (kt + kTileKeys > S) || (kt + kTileKeys > k1);
        bf16x8 pf[RPW][2];
#pragma unroll
        for (int rb = 0; rb < RPW; ++rb) {
            f32x16 s;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 a = __builtin_bit_cast(bf16x8, *(const u32x4*)&sK[col][ks * 16 + half * 8]);
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][ks], s, 0, 0, 0);
            }
            if (need_mask) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kabs = kt + 8 * (r >> 2) + 4 * half + (r & 3);
                    const bool vis = (kabs < S) || (kabs < k1 && ((mask[rb] >> ((kabs - S) & 63)) & 1ull));
                    s[r] = vis ? s[r] : -INFINITY;
                }
            }
            float mx = s[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m2[rb], mx * p.scale_log2);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new; // no visible key yet
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

        // ---- O^T += V^T . P^T
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) {
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const bf16x8 a =
                    __builtin_bit_cast(bf16x8, *(const u32x4*)&sVt[db * 32 + col][sl * 16 + half * 8]);
#pragma unroll
                for (int rb = 0; rb < RPW; ++rb)
                    acc[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[rb][sl], acc[rb][db], 0, 0, 0);
            }
        }
    }

    if (!wave_active) return;

    // ---- epilogue: lane (col, half) holds, for row `col`, channels db*32 + 8*(r/4) + 4*half + r%4
#pragma unroll
    for (int rb = 0; rb < RPW; ++rb) {
        const int r_local = row_base + rb * kRowBlock + col;
        const float l = lsum[rb] + __shfl_xor(lsum[rb], 32);
        if (r_local >= p.rows) continue;
        if (p.num_splits == 1) {
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
            const int64_t unit = (int64_t)b * p.Hkv + kvh;
            const int64_t prow = (unit * p.num_splits + split) * p.rows_pad + r_local;
            float* po = p.part_o + prow * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    f32x4 w = {acc[rb][db][4 * q4], acc[rb][db][4 * q4 + 1], acc[rb][db][4 * q4 + 2],
                               acc[rb][db][4 * q4 + 3]};
                    *(f32x4*)(po + db * 32 + 8 * q4 + 4 * half) = w;
                }
            if (half == 0) {
                p.part_ml[prow * 2] = m2[rb];
                p.part_ml[prow * 2 + 1] = l;
            }
        }
    }
}

// Merges the key splits of one query row: out = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
// grid = (ceil(rows / RPB), B * Hkv), block = 256: thread t owns 4 channels
// (t % (D/4)) of row t / (D/4) of its block of RPB = 1024 / D rows.
template <int D>
__global__ __launch_bounds__(256) void attn_combine_kernel(const AttnParams p) {
    constexpr int TPR = D / 4;      // threads per row
    constexpr int RPB = 256 / TPR;  // rows per block
    __shared__ int32_t sp[VS_MAX_TREE];
    __shared__ int32_t sflag;
    const int unit = blockIdx.y;
    const int b = unit / p.Hkv, kvh = unit % p.Hkv;
    const int32_t tree_code = load_tree(p.parent + (int64_t)b * p.T, p.T, sp, &sflag);
    const int32_t S = p.prefix_len[b];
    if (tree_code != VS_STATUS_OK || !prefix_ok(p, S)) return;
    const int row = blockIdx.x * RPB + threadIdx.x / TPR;
    const int ch = (threadIdx.x % TPR) * 4;
    if (row >= p.rows) return;
    const int nk = S + p.T;
    const int nsplit = min(p.num_splits, (nk + p.keys_per_split - 1) / p.keys_per_split);
    const int64_t base = (int64_t)unit * p.num_splits * p.rows_pad + row;
    float M = -INFINITY;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, p.part_ml[(base + (int64_t)s * p.rows_pad) * 2]);
    float den = 0.f;
    f32x4 num = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < nsplit; ++s) {
        const int64_t pr = base + (int64_t)s * p.rows_pad;
        const float ms = p.part_ml[pr * 2];
        if (ms == -INFINITY) continue; // this split saw no visible key for the row
        const float w = __builtin_amdgcn_exp2f(ms - M);
        den += w * p.part_ml[pr * 2 + 1];
        const f32x4 o = *(const f32x4*)(p.part_o + pr * D + ch);
        num += w * o;
    }
    const float inv = 1.f / den;
    const int node = row / p.group;
    const int hq = kvh * p.group + (row - node * p.group);
    uint16_t* o = (uint16_t*)p.out + (((int64_t)b * p.T + node) * p.Hq + hq) * D + ch;
    u32x2 w;
    w[0] = pack_bf16x2(num[0] * inv, num[1] * inv);
    w[1] = pack_bf16x2(num[2] * inv, num[3] * inv);
    *(u32x2*)o = w;
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
    const int rpb = 1024 / p.d;
    const dim3 grid((p.rows + rpb - 1) / rpb, p.B * p.Hkv);
    if (p.d == 128) hipLaunchKernelGGL((attn_combine_kernel<128>), grid, dim3(256), 0, s, p);
    else if (p.d == 64) hipLaunchKernelGGL((attn_combine_kernel<64>), grid, dim3(256), 0, s, p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

} // namespace vs
