// tf_decode_attn_full / tf_decode_attn_retrieval / tf_decode_attn_indexed / tf_decode_attn_tree:
// attention of G <= 16 speculated query tokens over a long bf16 KV cache (Algorithm 1: the
// M_p(C_p, ...) verification pass and the M_p(C_r, ...) drafting pass; the indexed form reads the
// draft cache through the chunk indices of Sec. 4.1 instead of a gathered copy; the tree form
// replaces the causal triangle over the G tokens by an ancestor mask, Sec. 5.3.3).
//
// Design (gfx950, wave64): flash-decoding. The KV sequence of every (b,h) is cut into
// `nsplit` contiguous ranges, one 256-thread workgroup each; its 4 waves walk interleaved
// 16-token tiles, so the workgroup streams K and V front to back. Per tile and wave:
//   * K rows arrive as MFMA A-operands (lane (r,s): token r, dims 32kk+8s..+8) and four
//     v_mfma_f32_16x16x32_bf16 give S^T[token, query] against the Q operand, which every wave
//     keeps in a private LDS slot and re-reads per tile (16 VGPRs fewer; no workgroup barrier);
//   * more than 4 query rows: the accumulator layout (lane (r,s), reg i = token 4s+i, query r) is
//     exactly the A-operand layout of v_mfma_f32_16x16x4_f32, so P = exp2(S - m) feeds the PV
//     product with no data movement; V rows arrive fully coalesced (lane (r,s): token 4s+i, dims
//     8r..8r+8), are widened bf16->fp32 in registers and serve as B-operands. P and V stay
//     fp32, so the only rounding is fp32 accumulation.
//   * up to 4 query rows (the draft pass): a 16-column MFMA would spend 32 x 32 matrix-pipe cycles
//     per tile on columns that are mostly zero queries, which is what bounds a short cache; here
//     every lane multiplies its own 4 tokens x 8 dims of V by the probabilities of each query row,
//     fetched from the lane that holds them by a row broadcast: 32 G FMAs per tile and lane.
//   * online softmax: the per-query running maximum is reduced over the tile with two
//     wave shuffles; accumulators are rescaled only when a maximum actually grows.
//   * all K/V loads carry the nt bit: the cache is touched once per pass and must not displace
//     anything in L2 / the last-level cache (+15% bandwidth measured).
// Every wave writes its own partial (m, l, O); a small second kernel merges the 4 x nsplit partials of
// a unit by log-sum-exp and normalises. The host plans the splits so that, where batch x heads
// allows, exactly one workgroup runs per CU (see plan_splits).
// The 16 columns of the QK^T MFMA hold up to 16 query rows, so the query heads of a
// grouped-query KV head share its pass; head dim 128 or 64.
#include <atomic>
#include <type_traits>

#include "tf_common.hpp"

namespace tf {

constexpr int kTile = 16;    // tokens per MFMA tile
constexpr int kWaves = 4;    // waves per workgroup
// tiles in flight per wave. Measured at 128K context, one workgroup per CU: depth 2 305 us,
// depth 3 307 us, depth 4 307 us per layer -- the stream is not latency-bound, so the
// shallowest pipeline (fewest registers) is used.
constexpr int kPipeDepth = 2;

struct AttnParams {
    const uint16_t *Q, *K, *V;
    int64_t sb, sh, st;
    const int32_t *kv_len;
    int32_t kv_len_all;  // plain: upper bound of the cache length; indexed: of the virtual length
    // G: query rows per KV head = (speculated tokens) x (query heads per KV head), <= 16: they are
    // the columns of the QK^T MFMA, so grouped-query heads ride along for free. Row r is token
    // r % Gm of query head r / Gm of the group; Gm = speculated tokens.
    int32_t H, G, Gm;
    // masked != 0: the last G tokens of the sequence are the queries' own; query g sees the
    // tokens before them and the j-th of them iff bit j of row g of tail_mask is set (causal:
    // bits 0..g; a token tree: the node's ancestors and itself). masked == 0: every query sees all.
    int32_t masked;
    uint64_t tail_mask[4];  // 16 rows of 16 bits
    int32_t nsplit, tokens_per_split;
    float scale_log2;
    float *part_o;   // [BH][nsplit * 4 waves][rows][head dim], rows = 8 or 16 (the kernel's kRows)
    float *part_ml;  // [BH][nsplit * 4 waves][2][rows]   (running max in log2 units, then sum)
    // indexed mode only: the virtual sequence of (b,h) is the chunks idx[b,h,0..k_chunks) of the
    // cache (chunk j = rows idx*chunk .. idx*chunk+chunk-1, negative entries skipped) followed
    // by the cache rows [recent_begin, len)
    const int32_t *idx;
    int32_t k_chunks, chunk;
    const int32_t *recent_begin;
    int32_t recent_begin_all;
    int32_t full_len_all;  // upper bound of the real cache length (rows that may be read)
};

__device__ __forceinline__ float safe_max(float m) { return m == -INFINITY ? 0.0f : m; }

// value of lane kSrc of this lane's row of 16 lanes (DPP row broadcast; no LDS traffic)
template <int kSrc>
__device__ __forceinline__ float row_bcast(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x150 + kSrc, 0xf,
                                                                 0xf, false));
}

constexpr int kValuRows = 4;  // most query rows the vector-ALU form of the PV product takes

// kD = head dim (128, or 64 for the small draft model's cache): kD/32 K loads and bf16 MFMAs per
// tile, kD/16 output dims (accumulators) per lane. kValu: at most kValuRows query rows, PV on the
// vector ALU (see the file comment).
template <bool kIndexed, int kDepth, int kD, int kRows, bool kValu>
__global__ __launch_bounds__(256) void attn_split_kernel(const AttnParams p) {
    constexpr int kNK = kD / 32;
    constexpr int kNE = kD / 16;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform by construction
    const int r = lane & 15, s = lane >> 4;
    const int split = blockIdx.x % p.nsplit;
    const int bh = blockIdx.x / p.nsplit;
    const int b = bh / p.H, h = bh - b * p.H;

    // len: number of (virtual) tokens of this sequence
    int len, rb = 0;
    const int kc_tokens = kIndexed ? p.k_chunks * p.chunk : 0;
    if constexpr (kIndexed) {
        int full = p.kv_len ? p.kv_len[b] : p.full_len_all;
        full = min(max(full, 0), p.full_len_all);
        rb = p.recent_begin ? p.recent_begin[b] : p.recent_begin_all;
        rb = min(max(rb, p.recent_begin_all), full);      // never below the promised lower bound
        len = min(kc_tokens + (full - rb), p.kv_len_all);
    } else {
        len = p.kv_len ? p.kv_len[b] : p.kv_len_all;
        len = min(max(len, 0), p.kv_len_all);
    }
    const int64_t tb64 = (int64_t)split * p.tokens_per_split;
    const int t_begin = (int)(tb64 < (int64_t)len ? tb64 : (int64_t)len);
    const int t_end = (int)(tb64 + p.tokens_per_split < (int64_t)len ? tb64 + p.tokens_per_split : (int64_t)len);
    const int last_row = max(len - 1, 0);

    // uniform base pointers + 32-bit per-lane byte offsets (scalar-base addressing)
    const char *Kb = reinterpret_cast<const char *>(p.K + (int64_t)b * p.sb + (int64_t)h * p.sh);
    const char *Vb = reinterpret_cast<const char *>(p.V + (int64_t)b * p.sb + (int64_t)h * p.sh);
    const int64_t row_bytes = p.st * 2;
    const uint32_t k_off = (uint32_t)(r * row_bytes + s * 16);  // K: token r, dims 8s.. (+64 B per kk)
    uint32_t v_off[4];                                          // V: token 4s+i, dims kNE*r..
#pragma unroll
    for (int i = 0; i < 4; ++i) v_off[i] = (uint32_t)((4 * s + i) * row_bytes + r * (kNE * 2));
    // one lane's share of a V row: 16 bytes (head dim 128) or 8 bytes (64, upper half unused)
    auto ldv = [](const void *ptr) -> uint4 {
        if constexpr (kD == 128) {
            return ld16_stream(ptr);
        } else {
            const uint2 h = ld8_stream(ptr);
            return make_uint4(h.x, h.y, 0u, 0u);
        }
    };

    // Q operand of the QK^T MFMAs, kept in LDS (re-read per tile: 4 KiB per tile is nothing for
    // LDS, and the lane has 16 VGPRs more for loads in flight): entry [kk][lane] holds
    // Q[query r][32kk + 8s .. +8] for lane (r,s), zero for r >= G
    // Every wave keeps a copy of its own: a lane reads back only what it wrote itself, so no
    // barrier stands between the start of the kernel and the first K/V loads.
    __shared__ uint4 sm_q[kWaves][kNK][kWave];
    // indexed mode: the chunk indices this split walks, staged once (a global index load in front
    // of every row load would put two memory latencies in series per tile)
    constexpr int kIdxStage = kIndexed ? 1024 : 1;
    __shared__ int32_t sm_idx[kIdxStage];
    const int j_first = kIndexed ? t_begin / p.chunk : 0;  // first chunk slot of this split
    if constexpr (kIndexed) {
        const int j_end = min(p.k_chunks, (t_end + p.chunk - 1) / p.chunk);
        for (int j = j_first + tid; j < min(j_end, j_first + kIdxStage); j += 256)
            sm_idx[j - j_first] = p.idx[(int64_t)bh * p.k_chunks + j];
    }
    // The Q loads are requested here, all at once and without a branch (rows past G read row G-1 and
    // are zeroed on the way to LDS); the LDS write, which has to wait for them, comes after the
    // first K/V requests are out, so one memory latency covers Q, K and V together.
    uint4 qv[kNK];
    {
        const uint16_t *qp = p.Q + ((int64_t)bh * p.G + min(r, p.G - 1)) * kD + s * 8;
#pragma unroll
        for (int kk = 0; kk < kNK; ++kk) qv[kk] = ld16(qp + kk * 32);
    }
    auto stage_q = [&]() {
#pragma unroll
        for (int kk = 0; kk < kNK; ++kk) sm_q[wave][kk][lane] = r < p.G ? qv[kk] : make_uint4(0, 0, 0, 0);
    };
    if constexpr (kIndexed) __syncthreads();  // the staged indices are shared by the workgroup

    // tokens < n_all are visible to every query; of the last G tokens this lane's query sees
    // those whose bit is set in my_mask
    const int n_all = p.masked ? len - p.Gm : len;
    const int my_row = r % p.Gm;  // this lane's query token
    const uint64_t my_word = my_row < 8 ? (my_row < 4 ? p.tail_mask[0] : p.tail_mask[1])
                                        : (my_row < 12 ? p.tail_mask[2] : p.tail_mask[3]);
    const uint32_t my_mask = (uint32_t)(my_word >> (16 * (my_row & 3))) & 0xffffu;

    // MFMA form: o[e][j] = O[query 4s+j][dim kNE*r+e]; vector-ALU form: ov[g][e] = this lane's share
    // (its tokens 4s..4s+3 of every tile) of O[query g][dim kNE*r+e]
    f32x4_t o[kValu ? 1 : kNE];
    float ov[kValu ? kValuRows : 1][kNE];
#pragma unroll
    for (int e = 0; e < (kValu ? 1 : kNE); ++e) o[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int g = 0; g < (kValu ? kValuRows : 1); ++g)
#pragma unroll
        for (int e = 0; e < kNE; ++e) ov[g][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // indexed mode: cache row of virtual token v, or -1 if it does not exist
    auto virtual_row = [&](int v) -> int {
        int row = -1;
        if (v < kc_tokens) {
            const int j = v / p.chunk;
            const int m = j - j_first < kIdxStage ? sm_idx[j - j_first] : p.idx[(int64_t)bh * p.k_chunks + j];
            if (m >= 0 && (int64_t)(m + 1) * p.chunk <= (int64_t)p.full_len_all) row = m * p.chunk + (v - j * p.chunk);
        } else if (v < len) {
            row = rb + (v - kc_tokens);
        }
        return row;
    };

    // loads of one tile; `rows` (indexed mode) is this lane's row for token t0+r, -1 = masked.
    // A tile that is not `live` (software-pipeline slots past the wave's last tile) is loaded
    // from one fixed valid location with all lanes on the same 16 bytes, so the number of loads
    // in flight never depends on control flow and the dummy costs one 64-byte request.
    auto load_k = [&](int t0, bool live, uint4(&k)[kNK], int &rows) {
        if constexpr (kIndexed) {
            rows = live ? virtual_row(t0 + r) : -1;
            const char *kp = Kb + (int64_t)max(rows, 0) * row_bytes + s * 16;
#pragma unroll
            for (int kk = 0; kk < kNK; ++kk) k[kk] = ld16_stream(kp + kk * 64);
        } else {
            const char *base = Kb + (int64_t)(live ? t0 : t_begin) * row_bytes;
            const uint32_t off = live ? k_off : 0u;
#pragma unroll
            for (int kk = 0; kk < kNK; ++kk) k[kk] = ld16_stream(base + off + kk * 64);
        }
    };
    // returns (indexed mode) the 4-bit validity mask of this lane's tokens 4s+i
    auto load_v = [&](int t0, bool live, uint4(&v)[4], int rows) -> int {
        int vm = 0xf;
        if constexpr (kIndexed) {
            vm = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int rv = __shfl(rows, 4 * s + i, kWave);   // row of token 4s+i (held by lane r'=4s+i)
                vm |= (rv >= 0) << i;
                v[i] = ldv(Vb + (int64_t)max(rv, 0) * row_bytes + r * (kNE * 2));
            }
        } else {
            const char *base = Vb + (int64_t)(live ? t0 : t_begin) * row_bytes;
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = ldv(base + (live ? v_off[i] : 0u));
        }
        return vm;
    };

    // S^T tile: four bf16 MFMAs over the head dim, then the log2-domain scale
    auto qk_tile = [&](const uint4(&k)[kNK], float(&z)[4]) {
        f32x4_t sc = f32x4_t{0.f, 0.f, 0.f, 0.f};
        asm volatile("" ::: "memory");  // keep the Q reads inside the loop (not hoisted into registers)
        uint4 qb[kNK];
#pragma unroll
        for (int kk = 0; kk < kNK; ++kk) qb[kk] = sm_q[wave][kk][lane];
#pragma unroll
        for (int kk = 0; kk < kNK; ++kk)
            sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, k[kk]),
                                                         __builtin_bit_cast(bf16x8_t, qb[kk]), sc, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) z[i] = sc[i] * p.scale_log2;
    };

    // online softmax of one tile and the P.V product
    auto softmax_pv = [&](int t0, float(&z)[4], const uint4(&v)[4], int vm) {
        if (kIndexed || t0 + kTile > n_all) {  // wave-uniform: tiles touching the causal / ragged tail
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int t = t0 + 4 * s + i;
                const bool visible = t < n_all || (t < len && ((my_mask >> ((t - n_all) & 31)) & 1u));
                if (!visible || !((vm >> i) & 1)) z[i] = -INFINITY;
            }
        }
        float mt = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
        mt = wave_max_xor(mt, 16);
        mt = wave_max_xor(mt, 32);
        const float m_new = fmaxf(m_run, mt);
        if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {  // some query's maximum grew
            const float alpha = __builtin_amdgcn_exp2f(m_run - safe_max(m_new));
            l_run *= alpha;
            if constexpr (kValu) {
                const float a4[kValuRows] = {row_bcast<0>(alpha), row_bcast<1>(alpha), row_bcast<2>(alpha),
                                             row_bcast<3>(alpha)};  // factor of query g: held by lane g of the row
#pragma unroll
                for (int g = 0; g < kValuRows; ++g)
#pragma unroll
                    for (int e = 0; e < kNE; ++e) ov[g][e] *= a4[g];
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float aj = __shfl(alpha, 4 * s + j, kWave);  // factor of query 4s+j
#pragma unroll
                    for (int e = 0; e < kNE; ++e) o[e][j] *= aj;
                }
            }
            m_run = m_new;
        }
        const float ms = safe_max(m_run);
        float pr[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) pr[i] = __builtin_amdgcn_exp2f(z[i] - ms);
        l_run += (pr[0] + pr[1]) + (pr[2] + pr[3]);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
            if constexpr (kValu) {
                // pr[i] of lane (g, s) is the weight of token 4s+i for query g: bring it to every
                // lane of the row, multiply this lane's kNE dims of that token's V row
                const float pg[kValuRows] = {row_bcast<0>(pr[i]), row_bcast<1>(pr[i]), row_bcast<2>(pr[i]),
                                             row_bcast<3>(pr[i])};
#pragma unroll
                for (int e = 0; e < kNE; ++e) {
                    const float vf = (e & 1) ? bf16hi(w[e >> 1]) : bf16lo(w[e >> 1]);
#pragma unroll
                    for (int g = 0; g < kValuRows; ++g) ov[g][e] = fmaf(pg[g], vf, ov[g][e]);
                }
            } else {
#pragma unroll
                for (int e = 0; e < kNE; ++e) {
                    const float vf = (e & 1) ? bf16hi(w[e >> 1]) : bf16lo(w[e >> 1]);
                    o[e] = __builtin_amdgcn_mfma_f32_16x16x4f32(pr[i], vf, o[e], 0, 0, 0);
                }
            }
        }
    };

    // 16-token tiles of this split, interleaved over the 4 waves, in a software pipeline of
    // kDepth tiles per wave: K of tile i+kDepth-1 is requested before the QK^T of tile i, its V
    // right after (when the K registers of tile i are dead). Loads are never conditional (see
    // load_k), so the wait counters stay exact. Plain mode walks whole tiles here and leaves a
    // ragged last tile to the clamped path below; indexed mode masks per token anyway, so the
    // ragged tile is just one more tile.
    const int n_full = kIndexed ? (t_end - t_begin + kTile - 1) / kTile : (t_end - t_begin) / kTile;
    const int n_mine_tiles = (n_full - wave + kWaves - 1) / kWaves;
    if (n_mine_tiles > 0) {
        constexpr int step = kWaves * kTile;
        uint4 kb[kDepth][kNK], vb[kDepth][4];
        int rws[kDepth], vms[kDepth];
        float z[4];
        const int t_first = t_begin + wave * kTile;
#pragma unroll
        for (int j = 0; j < kDepth - 1; ++j) {
            load_k(t_first + j * step, j < n_mine_tiles, kb[j], rws[j]);
            vms[j] = load_v(t_first + j * step, j < n_mine_tiles, vb[j], rws[j]);
        }
        stage_q();
        for (int i = 0; i < n_mine_tiles; i += kDepth) {
#pragma unroll
            for (int j = 0; j < kDepth; ++j) {
                const int nb = (j + kDepth - 1) % kDepth;   // buffer freed by the previous tile
                const int nxt = i + j + kDepth - 1;
                const bool cur_live = i + j < n_mine_tiles;
                load_k(t_first + nxt * step, nxt < n_mine_tiles, kb[nb], rws[nb]);
                if (cur_live) qk_tile(kb[j], z);
                vms[nb] = load_v(t_first + nxt * step, nxt < n_mine_tiles, vb[nb], rws[nb]);
                if (cur_live) softmax_pv(t_first + (i + j) * step, z, vb[j], vms[j]);
            }
        }
    }
    // plain mode, ragged tail (len not a multiple of 16): one partial tile, rows clamped to the
    // last valid token and masked; handled by the wave whose turn it would be
    if (!kIndexed && t_begin + n_full * kTile < t_end && (n_full % kWaves) == wave) {
        if (n_mine_tiles <= 0) stage_q();
        const int t0 = t_begin + n_full * kTile;
        uint4 kt[kNK], vt[4];
        float z[4];
        const char *kp = Kb + (int64_t)min(t0 + r, last_row) * row_bytes + s * 16;
#pragma unroll
        for (int kk = 0; kk < kNK; ++kk) kt[kk] = ld16_stream(kp + kk * 64);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            vt[i] = ldv(Vb + (int64_t)min(t0 + 4 * s + i, last_row) * row_bytes + r * (kNE * 2));
        qk_tile(kt, z);
        softmax_pv(t0, z, vt, 0xf);
    }

    // total of the per-lane partial sums of each query (lanes (r, 0..3))
    l_run += __shfl_xor(l_run, 16, kWave);
    l_run += __shfl_xor(l_run, 32, kWave);

    // every wave publishes its own partial: no LDS, no barrier; the merge kernel weighs them
    const int64_t pidx = ((int64_t)bh * p.nsplit + split) * kWaves + wave;
    float *po = p.part_o + pidx * kRows * kD;
    if (s == 0 && r < p.G) {
        p.part_ml[(pidx * 2 + 0) * kRows + r] = m_run;
        p.part_ml[(pidx * 2 + 1) * kRows + r] = l_run;
    }
    if constexpr (kValu) {
        // sum the four token groups (lanes (r, 0..3)), then lanes (r, 0) write dims kNE*r.. of each query
#pragma unroll
        for (int g = 0; g < kValuRows; ++g)
#pragma unroll
            for (int e = 0; e < kNE; ++e) {
                float t = ov[g][e];
                t += __shfl_xor(t, 16, kWave);
                t += __shfl_xor(t, 32, kWave);
                ov[g][e] = t;
            }
        if (s == 0) {
#pragma unroll
            for (int g = 0; g < kValuRows; ++g)
                if (g < p.G) {
                    float *dst = po + g * kD + kNE * r;
                    *reinterpret_cast<float4 *>(dst) = make_float4(ov[g][0], ov[g][1], ov[g][2], ov[g][3]);
                    if constexpr (kNE == 8)
                        *reinterpret_cast<float4 *>(dst + 4) = make_float4(ov[g][4], ov[g][5], ov[g][6], ov[g][7]);
                }
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (4 * s + j < p.G) {
                float *dst = po + (4 * s + j) * kD + kNE * r;
                *reinterpret_cast<float4 *>(dst) = make_float4(o[0][j], o[1][j], o[2][j], o[3][j]);
                if constexpr (kNE == 8)
                    *reinterpret_cast<float4 *>(dst + 4) = make_float4(o[4][j], o[5][j], o[6][j], o[7][j]);
            }
    }
}

// Merge of few partials (at most kP, a template constant), one 128- or 64-thread workgroup per
// (b,h,g), thread = output dim. No LDS and no barrier: the maxima and sums of the partials are read
// with wave-uniform addresses, the kP partial values of this thread's dim are all requested before
// the first is used, so the whole merge costs about one memory round trip.
template <int kD, int kP>
__global__ __launch_bounds__(kD) void attn_combine_small_kernel(const float *__restrict__ part_o,
                                                                const float *__restrict__ part_ml, int nparts,
                                                                int G, int rows, float *__restrict__ O,
                                                                float *__restrict__ LSE) {
    const int dim = threadIdx.x;
    const int bh = blockIdx.x / G, g = blockIdx.x - bh * G;
    const int64_t base = (int64_t)bh * nparts;
    const float *po = part_o + (base * rows + g) * kD + dim;
    const float *pm = part_ml + base * 2 * rows + g;
    const int64_t stride_o = (int64_t)rows * kD, stride_ml = 2 * rows;
    float ov[kP], mv[kP], lv[kP];
#pragma unroll
    for (int sp = 0; sp < kP; ++sp) {
        const int q = sp < nparts ? sp : 0;        // past the end: partial 0 again, weight 0 below
        ov[sp] = po[q * stride_o];
        mv[sp] = sp < nparts ? pm[q * stride_ml] : -INFINITY;
        lv[sp] = pm[q * stride_ml + rows];
    }
    float M = -INFINITY;
#pragma unroll
    for (int sp = 0; sp < kP; ++sp) M = fmaxf(M, mv[sp]);
    const float Ms = safe_max(M);
    float L = 0.f, acc = 0.f;
#pragma unroll
    for (int sp = 0; sp < kP; ++sp) {
        const float a = __builtin_amdgcn_exp2f(mv[sp] - Ms);   // exp2(-inf) = 0 for empty and padded partials
        L = fmaf(a, lv[sp], L);
        acc = fmaf(a, ov[sp], acc);
    }
    const int64_t row = (int64_t)bh * G + g;
    O[row * kD + dim] = L > 0.f ? acc / L : 0.f;
    if (LSE && dim == 0) LSE[row] = L > 0.f ? (M + __log2f(L)) * kLn2 : -INFINITY;
}

// Merge of many partials of one (b,h,g) (`nsplit` below counts partials: 4 per split). 512 threads
// = 4 groups x 128 output dims. The per-partial maxima and sums are staged in LDS, turned into
// weights once, and each group accumulates every 4th partial with independent loads in flight;
// groups are summed in LDS.
constexpr int kCombineThreads = 512;
constexpr int kMaxParts = 2048;               // partials the merge kernel stages weights for
constexpr int kMaxSplits = kMaxParts / kWaves;
constexpr int kSmallParts = 32;               // up to here the barrier-free merge is used (more would spill scalar registers)

template <int kD>
__global__ __launch_bounds__(kCombineThreads) void attn_combine_kernel(const float *__restrict__ part_o,
                                                                       const float *__restrict__ part_ml,
                                                                       int nsplit, int G, int rows,
                                                                       float *__restrict__ O,
                                                                       float *__restrict__ LSE) {
    __shared__ float sm_w[kMaxParts];   // running max, then weight exp2(m - M), per partial
    __shared__ float sm_l[kMaxParts];
    __shared__ float sm_red[kCombineThreads / 64];
    constexpr int kCombineGroups = kCombineThreads / kD;
    __shared__ float sm_acc[kCombineGroups][kD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bh = blockIdx.x / G, g = blockIdx.x - bh * G;
    const int64_t base = (int64_t)bh * nsplit;

    float mx = -INFINITY;
    for (int sp = tid; sp < nsplit; sp += kCombineThreads) {
        const float m = part_ml[((base + sp) * 2 + 0) * rows + g];
        sm_w[sp] = m;
        sm_l[sp] = part_ml[((base + sp) * 2 + 1) * rows + g];
        mx = fmaxf(mx, m);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = wave_max_xor(mx, off);
    if (lane == 0) sm_red[wave] = mx;
    __syncthreads();
    float M = sm_red[0];
#pragma unroll
    for (int w = 1; w < kCombineThreads / 64; ++w) M = fmaxf(M, sm_red[w]);
    const float Ms = safe_max(M);
    float lpart = 0.f;
    for (int sp = tid; sp < nsplit; sp += kCombineThreads) {
        const float a = __builtin_amdgcn_exp2f(sm_w[sp] - Ms);
        sm_w[sp] = a;
        lpart += a * sm_l[sp];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) lpart += __shfl_xor(lpart, off, kWave);
    __syncthreads();  // sm_red is reused; weights become visible
    if (lane == 0) sm_red[wave] = lpart;
    __syncthreads();
    float L = 0.f;
#pragma unroll
    for (int w = 0; w < kCombineThreads / 64; ++w) L += sm_red[w];

    const int dim = tid % kD, grp = tid / kD;
    const float *po = part_o + (base * rows + g) * kD + dim;
    const int64_t split_stride = (int64_t)rows * kD;
    float acc = 0.f;
    int sp = grp;
    for (; sp + 3 * kCombineGroups < nsplit; sp += 4 * kCombineGroups) {
        const float v0 = po[(int64_t)sp * split_stride];
        const float v1 = po[(int64_t)(sp + kCombineGroups) * split_stride];
        const float v2 = po[(int64_t)(sp + 2 * kCombineGroups) * split_stride];
        const float v3 = po[(int64_t)(sp + 3 * kCombineGroups) * split_stride];
        acc += sm_w[sp] * v0;
        acc += sm_w[sp + kCombineGroups] * v1;
        acc += sm_w[sp + 2 * kCombineGroups] * v2;
        acc += sm_w[sp + 3 * kCombineGroups] * v3;
    }
    for (; sp < nsplit; sp += kCombineGroups) acc += sm_w[sp] * po[(int64_t)sp * split_stride];
    sm_acc[grp][dim] = acc;
    __syncthreads();
    if (tid < kD) {
        float tot = sm_acc[0][tid];
#pragma unroll
        for (int q = 1; q < kCombineGroups; ++q) tot += sm_acc[q][tid];
        const int64_t row = (int64_t)bh * G + g;
        O[row * kD + tid] = L > 0.f ? tot / L : 0.f;
        if (LSE && tid == 0) LSE[row] = L > 0.f ? (M + __log2f(L)) * kLn2 : -INFINITY;
    }
}

struct SplitPlan {
    int nsplit;
    int tokens_per_split;
};

// Tokens per split, 0 = automatic. A process-wide default (atomic: may be set while other threads
// call) and a per-thread override (-1 = none) that only the calling thread's later queries and
// calls see, so two host threads driving two streams can tune independently.
static std::atomic<int64_t> g_tps_full{0}, g_tps_retr{0};
static thread_local int64_t t_tps_full = -1, t_tps_retr = -1;

int set_attn_option(bool retrieval, int64_t v, bool this_thread) {
    if (this_thread && v == -1) {
        (retrieval ? t_tps_retr : t_tps_full) = -1;
        return TF_OK;
    }
    if (v < 0 || (v % 64) != 0 || v > (1 << 30)) return TF_ERR_INVALID_ARG;
    if (this_thread) (retrieval ? t_tps_retr : t_tps_full) = v;
    else (retrieval ? g_tps_retr : g_tps_full).store(v, std::memory_order_relaxed);
    return TF_OK;
}

static int64_t tps_option(bool retrieval) {
    const int64_t t = retrieval ? t_tps_retr : t_tps_full;
    return t >= 0 ? t : (retrieval ? g_tps_retr : g_tps_full).load(std::memory_order_relaxed);
}

// compute units of the current device (256 on a full MI355X), queried once per device
static int num_cus() {
    constexpr int kMaxDevices = 64;
    static std::atomic<int> cached[kMaxDevices];  // zero-initialised; 0 = not asked yet
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// Split planning. Measured on MI355X with streaming (nt) loads: the fewer workgroups stream
// concurrently, the higher the HBM bandwidth, as long as every CU has one -- at 128K context one
// workgroup per CU reads 7.05 TB/s, two per CU 6.90, three per CU 6.70 (fewer DRAM streams in
// flight); a count that leaves CUs with unequal numbers of workgroups is far worse (1.5 per CU:
// 5.7 TB/s), and so are unequal splits. The plan therefore takes, among the split counts whose
// splits are equal, the one with the smallest modelled time
//     (workgroups on the busiest CU) x (tokens per split) / rate(workgroups per CU),
// which is "one workgroup per CU" whenever batch x heads divides the CU count.
// The indexed form reads scattered chunks (a few KiB each) instead of one long stream, so it is
// latency-bound and wants the opposite: three workgroups per CU (19 us against 23.5 us per layer at
// a 4K budget).
enum PlanMode { kPlanFull = 0, kPlanRetrieval = 1, kPlanIndexed = 2 };
// shorter splits are all overhead
static int64_t min_tokens_per_split(PlanMode mode) { return mode != kPlanFull ? 128 : 512; }

static SplitPlan plan_splits(int64_t BH, int64_t kv_len_all, PlanMode mode) {
    const bool retrieval = mode != kPlanFull;
    int64_t tps = tps_option(retrieval);
    if (tps == 0) {
        struct Memo {
            int64_t BH, len, cus;
            int64_t tps;
        };
        static thread_local Memo memo[3] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
        Memo &mm = memo[mode];
        const int64_t cus = num_cus();
        if (mm.BH == BH && mm.len == kv_len_all && mm.cus == cus) {
            tps = mm.tps;
        } else {
            int64_t ns_cap = kv_len_all / min_tokens_per_split(mode);
            if (ns_cap > kMaxSplits) ns_cap = kMaxSplits;   // the merge kernel stages one weight per split
            const int64_t ns_useful = (8 * cus + BH - 1) / BH;  // beyond 8 workgroups per CU nothing changes
            if (ns_cap > ns_useful) ns_cap = ns_useful;
            if (ns_cap < 1) ns_cap = 1;
            double best = 0.0;
            for (int64_t ns = 1; ns <= ns_cap; ++ns) {
                // whole 16-token tiles per split (the 4 waves interleave tiles, so any tile count balances
                // them to within one tile)
                const int64_t t = (((kv_len_all + ns - 1) / ns + kTile - 1) / kTile) * kTile;
                const int64_t n_eff = (kv_len_all + t - 1) / t;
                const int64_t per_cu = (BH * n_eff + cus - 1) / cus;
                const double rate = mode == kPlanIndexed ? (per_cu <= 1 ? 0.80 : (per_cu == 2 ? 0.95 : 1.0))
                                                         : (per_cu <= 1 ? 1.0 : (per_cu == 2 ? 0.982 : 0.955));
                const double cost = (double)per_cu * (double)t / rate;
                if (ns == 1 || cost < best * (1.0 - 1e-9)) {
                    best = cost;
                    tps = t;
                }
            }
            mm.BH = BH;
            mm.len = kv_len_all;
            mm.cus = cus;
            mm.tps = tps;
        }
    }
    int64_t ns = (kv_len_all + tps - 1) / tps;
    if (ns > kMaxSplits) {
        tps = (((kv_len_all + kMaxSplits - 1) / kMaxSplits + 63) / 64) * 64;
        ns = (kv_len_all + tps - 1) / tps;
    }
    if (ns < 1) ns = 1;
    return SplitPlan{(int)ns, (int)tps};
}

// sized for head dim 128 whatever the call's head dim (the queries do not take it); 8 query rows per
// KV head, 16 when there are more than 8
static int rows_of(int G) { return G > 8 ? 16 : 8; }
static size_t attn_ws_bytes(int64_t BH, int64_t nsplit, int G) {  // one partial per wave of every split
    return (size_t)BH * nsplit * kWaves * (rows_of(G) * kHeadDim + 2 * rows_of(G)) * sizeof(float);
}

// The most splits any call with a length in [1, len_bound] can plan under the options in force.
// The planned count itself is not monotone in the length (it snaps to counts that fill the CUs
// evenly), so the workspace queries size for this bound: a workspace queried for some length then
// serves every call with that length or less.
static int64_t max_splits_upto(int64_t BH, int64_t len_bound, PlanMode mode) {
    const bool retrieval = mode != kPlanFull;
    const int64_t tps = tps_option(retrieval);
    int64_t ns;
    if (tps > 0) {
        ns = (len_bound + tps - 1) / tps;
    } else {
        ns = len_bound / min_tokens_per_split(mode);
        const int64_t ns_useful = (8 * (int64_t)num_cus() + BH - 1) / BH;
        if (ns > ns_useful) ns = ns_useful;
    }
    if (ns > kMaxSplits) ns = kMaxSplits;
    return ns < 1 ? 1 : ns;
}

// the launch shape a call with these sizes would take now (for callers that want to know, and tests)
int attn_plan(int32_t kind, int32_t batch, int32_t heads, int64_t len_all, int32_t *nsplit, int32_t *tokens_per_split) {
    if (kind < 0 || kind > 2 || batch <= 0 || heads <= 0 || len_all <= 0 || !nsplit || !tokens_per_split)
        return TF_ERR_INVALID_ARG;
    if (len_all > (int64_t)1 << 30) return TF_ERR_UNSUPPORTED;
    const SplitPlan sp = plan_splits((int64_t)batch * heads, len_all, (PlanMode)kind);
    *nsplit = sp.nsplit;
    *tokens_per_split = sp.tokens_per_split;
    return TF_OK;
}

size_t attn_workspace_bytes(int32_t batch, int32_t heads, int64_t kv_len_all, int32_t G, bool retrieval) {
    if (batch <= 0 || heads <= 0 || kv_len_all <= 0 || G <= 0) return 0;
    const int64_t BH = (int64_t)batch * heads;
    return attn_ws_bytes(BH, max_splits_upto(BH, kv_len_all, retrieval ? kPlanRetrieval : kPlanFull), G);
}


static int64_t virtual_len_all(const IndexedArgs &ix, int64_t kv_len_all) {
    return (int64_t)ix.k_chunks * ix.chunk + (kv_len_all - ix.recent_begin_all);
}

size_t attn_indexed_workspace_bytes(int32_t batch, int32_t heads, int32_t k_chunks, int32_t chunk,
                                    int64_t recent_len_all, int32_t G) {
    if (batch <= 0 || heads <= 0 || k_chunks < 0 || chunk <= 0 || recent_len_all < 0 || G <= 0) return 0;
    const int64_t lv = (int64_t)k_chunks * chunk + recent_len_all;
    if (lv <= 0) return 0;
    const int64_t BH = (int64_t)batch * heads;
    return attn_ws_bytes(BH, max_splits_upto(BH, lv, kPlanIndexed), G);
}

int attn_launch(const void *Q, const void *K, const void *V, const tf_kv_desc *kd, const int32_t *kv_len,
                int64_t kv_len_all, int32_t G, float scale, int32_t causal, float *O, float *LSE, void *ws,
                size_t ws_bytes, void *stream, bool retrieval, const IndexedArgs *ix, const uint16_t *tail_mask) {
    if (!Q || !K || !V || !O) return TF_ERR_INVALID_ARG;
    int rc = check_desc(kd, true);
    if (rc != TF_OK) return rc;
    if (G < 1 || kd->q_group < 0) return TF_ERR_INVALID_ARG;
    if (G > TF_MAX_QUERIES) return TF_ERR_UNSUPPORTED;
    const int q_group = kd->q_group > 0 ? kd->q_group : 1;  // query heads per KV head
    if ((int64_t)G * q_group > 16) return TF_ERR_UNSUPPORTED; // the rows are the 16 columns of one MFMA
    const int GQ = G * q_group;
    if (kv_len_all < 1 || kv_len_all > kd->capacity) return TF_ERR_INVALID_ARG;
    if (kd->capacity > (int64_t)1 << 30 || kd->stride_t > (1 << 24)) return TF_ERR_UNSUPPORTED;
    int64_t plan_len = kv_len_all;  // length the splits are planned on
    if (ix) {
        if (ix->k_chunks < 0 || ix->chunk < 1 || (ix->k_chunks > 0 && !ix->idx)) return TF_ERR_INVALID_ARG;
        if (ix->chunk > 64) return TF_ERR_UNSUPPORTED;
        if (ix->recent_begin_all < 0 || ix->recent_begin_all > kv_len_all) return TF_ERR_INVALID_ARG;
        if (causal && kv_len_all - ix->recent_begin_all < G) return TF_ERR_INVALID_ARG;  // queries are recent rows
        plan_len = virtual_len_all(*ix, kv_len_all);
        if (plan_len < 1) return TF_ERR_INVALID_ARG;
        if (plan_len > (int64_t)1 << 30) return TF_ERR_UNSUPPORTED;
    }
    if ((causal || tail_mask) && plan_len < G) return TF_ERR_INVALID_ARG;
    if (!(scale == scale) || scale - scale != 0.f) return TF_ERR_INVALID_ARG;  // NaN or infinite
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16)) return TF_ERR_INVALID_ARG;
    const int64_t BH = (int64_t)kd->batch * kd->heads;
    const SplitPlan sp = plan_splits(BH, plan_len, ix ? kPlanIndexed : (retrieval ? kPlanRetrieval : kPlanFull));
    if (BH * sp.nsplit >= (int64_t)1 << 31) return TF_ERR_UNSUPPORTED;
    if (!ws || !aligned(ws, 256) || ws_bytes < attn_ws_bytes(BH, sp.nsplit, GQ)) return TF_ERR_WORKSPACE;

    AttnParams p;
    p.Q = static_cast<const uint16_t *>(Q);
    p.K = static_cast<const uint16_t *>(K);
    p.V = static_cast<const uint16_t *>(V);
    p.sb = kd->stride_b;
    p.sh = kd->stride_h;
    p.st = kd->stride_t;
    p.kv_len = kv_len;
    p.kv_len_all = (int32_t)plan_len;
    p.H = kd->heads;
    p.G = GQ;
    p.Gm = G;
    p.masked = (causal || tail_mask) ? 1 : 0;
    for (int i = 0; i < 4; ++i) p.tail_mask[i] = 0;
    for (int g = 0; g < G; ++g) {
        const uint32_t row = tail_mask ? (tail_mask[g] & ((1u << G) - 1u)) : ((2u << g) - 1u);
        p.tail_mask[g >> 2] |= (uint64_t)row << (16 * (g & 3));
    }
    p.nsplit = sp.nsplit;
    p.tokens_per_split = sp.tokens_per_split;
    p.scale_log2 = scale * kLog2e;
    p.part_o = static_cast<float *>(ws);
    const int rows = rows_of(GQ);
    p.part_ml = p.part_o + (size_t)BH * sp.nsplit * kWaves * rows * kd->head_dim;
    p.idx = ix ? ix->idx : nullptr;
    p.k_chunks = ix ? ix->k_chunks : 0;
    p.chunk = ix ? ix->chunk : 1;
    p.recent_begin = ix ? ix->recent_begin : nullptr;
    p.recent_begin_all = ix ? (int32_t)ix->recent_begin_all : 0;
    p.full_len_all = (int32_t)kv_len_all;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)(BH * sp.nsplit));
    const dim3 cgrid((unsigned)(BH * GQ));
    const int nparts = sp.nsplit * kWaves;
    auto launch = [&](auto d_tag, auto rows_tag, auto valu_tag) {
        constexpr int kD = decltype(d_tag)::value, kRows = decltype(rows_tag)::value;
        constexpr bool kValu = decltype(valu_tag)::value;
        if (ix)
            hipLaunchKernelGGL((attn_split_kernel<true, kPipeDepth, kD, kRows, kValu>), grid, dim3(256), 0, st, p);
        else
            hipLaunchKernelGGL((attn_split_kernel<false, kPipeDepth, kD, kRows, kValu>), grid, dim3(256), 0, st, p);
        if (nparts <= 16)
            hipLaunchKernelGGL((attn_combine_small_kernel<kD, 16>), cgrid, dim3(kD), 0, st, p.part_o, p.part_ml, nparts,
                               GQ, kRows, O, LSE);
        else if (nparts <= kSmallParts)
            hipLaunchKernelGGL((attn_combine_small_kernel<kD, kSmallParts>), cgrid, dim3(kD), 0, st, p.part_o, p.part_ml,
                               nparts, GQ, kRows, O, LSE);
        else
            hipLaunchKernelGGL((attn_combine_kernel<kD>), cgrid, dim3(kCombineThreads), 0, st, p.part_o, p.part_ml,
                               nparts, GQ, kRows, O, LSE);
    };
    using std::integral_constant;
    using std::false_type;
    using std::true_type;
    if (kd->head_dim == 128) {
        if (GQ <= kValuRows) launch(integral_constant<int, 128>{}, integral_constant<int, 8>{}, true_type{});
        else if (rows == 8) launch(integral_constant<int, 128>{}, integral_constant<int, 8>{}, false_type{});
        else launch(integral_constant<int, 128>{}, integral_constant<int, 16>{}, false_type{});
    } else {
        if (GQ <= kValuRows) launch(integral_constant<int, 64>{}, integral_constant<int, 8>{}, true_type{});
        else if (rows == 8) launch(integral_constant<int, 64>{}, integral_constant<int, 8>{}, false_type{});
        else launch(integral_constant<int, 64>{}, integral_constant<int, 16>{}, false_type{});
    }
    return hip_status(hipGetLastError());
}

// ---- the entry point that allocates nothing ---------------------------------------------------
// For callers that cannot allocate (HIP graph capture, tight serving loops): the split partials of
// the draft attention live in a file-scope device array instead of a caller workspace. Every GPU
// holds its own copy of the array at its own address; the address is looked up once per device
// (with that device current) and only that pointer is ever handed to kernels. The array's name in
// host code is a stand-in for the symbol, not a device address.
constexpr size_t kScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kScratchBytes];
constexpr int kScratchMaxDevices = 64;
static std::atomic<void *> g_scratch_ptr[kScratchMaxDevices];  // zero-initialised: not looked up yet

static int scratch_of_current_device(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kScratchMaxDevices) return TF_ERR_HIP;
    void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return TF_ERR_HIP;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // racing threads store the same address
    }
    *out = ptr;
    return TF_OK;
}

int attn_noalloc_init() {
    void *ptr = nullptr;
    return scratch_of_current_device(&ptr);
}

size_t attn_noalloc_max_bytes() { return kScratchBytes; }

int attn_retrieval_noalloc_launch(const void *Q, const void *K, const void *V, const tf_kv_desc *kd,
                                  const int32_t *kv_len, int64_t kv_len_all, int32_t G, float scale, int32_t causal,
                                  float *O, float *LSE, void *stream) {
    // the size check comes first (host arithmetic and a cached attribute query only): a too-large
    // problem is refused the same way whether or not the scratch address has been looked up yet
    if (kd && kd->batch > 0 && kd->heads > 0 && kv_len_all > 0 && G > 0) {
        const int q_group = kd->q_group > 0 ? kd->q_group : 1;
        const int64_t BH = (int64_t)kd->batch * kd->heads;
        if (kv_len_all <= (int64_t)1 << 30) {  // (longer lengths are refused by the launch below)
            const size_t need = attn_ws_bytes(BH, plan_splits(BH, kv_len_all, kPlanRetrieval).nsplit, G * q_group);
            if (need > kScratchBytes) return TF_ERR_SCRATCH_LIMIT;
        }
    }
    void *ptr = nullptr;
    const int rc = scratch_of_current_device(&ptr);
    if (rc != TF_OK) return rc;
    return attn_launch(Q, K, V, kd, kv_len, kv_len_all, G, scale, causal, O, LSE, ptr, kScratchBytes, stream, true,
                       nullptr, nullptr);
}

}  // namespace tf
