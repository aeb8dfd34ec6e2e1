// tf_chunk_topk_gather: retrieval-cache construction (Sec. 4.1 / Sec. 4.3): score every
// chunk by query . average-key, keep the k best in descending order, gather their K/V.
//
// Two launch shapes on one stream. Few (b,h) units in the call (one layer): three kernels,
//   score   HBM streaming over the fp32 average-key table (512 B per chunk). A wave takes 16
//           chunk rows at a time, 8 lanes per row reading whole 128-byte lines; 32 fp32 FMAs
//           per lane against the resident query, three shuffles per row finish the dot product.
//   select  one 1024-thread workgroup per (b,h): exact radix select (4 x 8 bits, LDS
//           histograms) of the k-th largest order-preserving key, ordered compaction of the
//           winners (ties toward the lower chunk index), then every winner's place on
//           (score desc, index asc) by counting the winners above it in LDS.
//   gather  one wave per selected chunk copies its rows (256 B each) of K and V with 16-byte
//           loads and stores.
// Many units (all layers of a decode step in one call): score and select fused into one kernel,
// one workgroup per unit, the unit's score keys held in LDS (score_select_kernel below), then the
// same gather. Both shapes compute the same fp32 scores in the same order and return the same bits.
#include <atomic>
#include <type_traits>

#include "tf_common.hpp"

namespace tf {

constexpr int kScoreMaxIters = 16;  // 16-row steps per wave (a workgroup covers 4 x 16 x iters rows)
constexpr int kSelThreads = 1024;
// 16-row steps per wave of the scoring kernel, 0 = automatic: a process-wide default (atomic) and a
// per-thread override (-1 = none), as for the attention split options
static std::atomic<int64_t> g_score_iters{0};
static thread_local int64_t t_score_iters = -1;

int set_score_option(int64_t v, bool this_thread) {
    if (this_thread && v == -1) {
        t_score_iters = -1;
        return TF_OK;
    }
    if (v < 0 || v > 4096) return TF_ERR_INVALID_ARG;
    if (this_thread) t_score_iters = v;
    else g_score_iters.store(v, std::memory_order_relaxed);
    return TF_OK;
}
// fused scoring + selection: 0 = automatic, 1 = whenever the shape allows, 2 = never
static std::atomic<int64_t> g_fused{0};
static thread_local int64_t t_fused = -1;

int set_fused_option(int64_t v, bool this_thread) {
    if (this_thread && v == -1) {
        t_fused = -1;
        return TF_OK;
    }
    if (v < 0 || v > 2) return TF_ERR_INVALID_ARG;
    if (this_thread) t_fused = v;
    else g_fused.store(v, std::memory_order_relaxed);
    return TF_OK;
}
static int64_t fused_option() { return t_fused >= 0 ? t_fused : g_fused.load(std::memory_order_relaxed); }

static int64_t score_iters_option() {
    return t_score_iters >= 0 ? t_score_iters : g_score_iters.load(std::memory_order_relaxed);
}

// compute units of the current device (256 on a full MI355X; also the assumption without a device)
static int compute_units() {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
        return 256;
    return n;
}

struct ScoreParams {
    const uint16_t *q_r;
    const void *Kmean;  // fp32, or bf16 for the bf16 scoring kernel
    int64_t M_cap;
    const int32_t *n_chunks;
    int32_t n_all, H;
    int32_t blocks_per_bh, iters;
    float *scores;
    int64_t score_stride;
};

// Every load instruction of a wave reads 8 rows x 128 contiguous bytes (whole cache lines:
// 64-byte pieces stream about 9% slower): lane (e, w) = (lane % 8, lane / 8) holds dims
// {32j + 4e .. +4}, j < 4, of row w, does 16 fp32 FMAs against the resident query and three
// shuffles over the 8 lanes of a row finish the dot product. The next step's loads are in flight
// while the current one is reduced.
__global__ __launch_bounds__(256) void chunk_score_kernel(const ScoreParams p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int e = lane & 7, w = lane >> 3;
    const int blk = blockIdx.x % p.blocks_per_bh;
    const int64_t bh = blockIdx.x / p.blocks_per_bh;
    const int b = (int)(bh / p.H);
    int n = p.n_chunks ? p.n_chunks[b] : p.n_all;
    n = min(max(n, 0), p.n_all);
    const int last_row = max(n - 1, 0);

    float q[4][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint2 u = *reinterpret_cast<const uint2 *>(p.q_r + bh * kHeadDim + 32 * j + 4 * e);
        q[j][0] = bf16lo(u.x);
        q[j][1] = bf16hi(u.x);
        q[j][2] = bf16lo(u.y);
        q[j][3] = bf16hi(u.y);
    }
    const float *base = static_cast<const float *>(p.Kmean) + bh * p.M_cap * kHeadDim + 4 * e;
    float *out = p.scores + bh * p.score_stride;

    // the 4 waves interleave 16-row steps over the workgroup's contiguous range (one stream
    // per workgroup, as in the attention kernel)
    const int m_begin = blk * 64 * p.iters + wave * 16;
    const int m_end = min((blk + 1) * 64 * p.iters, p.n_all);
    int left = (m_end - m_begin + 63) / 64;  // 16-row steps of this wave

    // rows past the sequence's chunk count are clamped to its last row (read, never stored)
    auto load = [&](int m0, float4(&v)[8]) {
#pragma unroll
        for (int rr = 0; rr < 2; ++rr) {
            const float *row = base + (int64_t)min(m0 + 8 * rr + w, last_row) * kHeadDim;
#pragma unroll
            for (int j = 0; j < 4; ++j) v[4 * rr + j] = ldf4_stream(row + 32 * j);
        }
    };
    auto finish = [&](int m0, const float4(&v)[8]) {
        float acc[2];
#pragma unroll
        for (int rr = 0; rr < 2; ++rr) {
            float a = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                a = fmaf(q[j][0], v[4 * rr + j].x, a);
                a = fmaf(q[j][1], v[4 * rr + j].y, a);
                a = fmaf(q[j][2], v[4 * rr + j].z, a);
                a = fmaf(q[j][3], v[4 * rr + j].w, a);
            }
            a += __shfl_xor(a, 1, kWave);
            a += __shfl_xor(a, 2, kWave);
            a += __shfl_xor(a, 4, kWave);
            acc[rr] = a;
        }
        // lanes e = 0 / e = 1 store rows m0 + w / m0 + 8 + w. (These few stores cost 10-15% of
        // the stream's bandwidth -- 7.1 -> 6.2 TB/s in isolation -- whether written per step or
        // collected in LDS and written as one 4 KiB burst per workgroup; only scores that never
        // leave the L2 are free, so the simple form stays. As nt stores they cost 5% less.)
        const int m = m0 + 8 * e + w;
        if (e < 2 && m < p.n_all)
            __builtin_nontemporal_store(m < n ? (e == 0 ? acc[0] : acc[1]) : -INFINITY, &out[m]);
    };

    if (left > 0) {
        float4 va[8], vb[8];
        int m0 = m_begin;
        load(m0, va);
        while (left > 2) {
            load(m0 + 64, vb);
            finish(m0, va);
            load(m0 + 128, va);
            finish(m0 + 64, vb);
            m0 += 128;
            left -= 2;
        }
        if (left == 2) {
            load(m0 + 64, vb);
            finish(m0, va);
            finish(m0 + 64, vb);
        } else {
            finish(m0, va);
        }
    }
}

// The same scoring over a bf16 average-key table (256 B per chunk, half the traffic): 16 lanes per
// row, 4 whole rows per load instruction, lane (e, w) = (lane % 16, lane / 16) holds dims 8e..8e+8
// of row w, 8 fp32 FMAs on the widened values per load and four shuffles per row.
__global__ __launch_bounds__(256) void chunk_score_bf16_kernel(const ScoreParams p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int e = lane & 15, w = lane >> 4;
    const int blk = blockIdx.x % p.blocks_per_bh;
    const int64_t bh = blockIdx.x / p.blocks_per_bh;
    const int b = (int)(bh / p.H);
    int n = p.n_chunks ? p.n_chunks[b] : p.n_all;
    n = min(max(n, 0), p.n_all);
    const int last_row = max(n - 1, 0);

    float q[8];
    {
        const uint4 u = ld16(p.q_r + bh * kHeadDim + 8 * e);
        q[0] = bf16lo(u.x); q[1] = bf16hi(u.x); q[2] = bf16lo(u.y); q[3] = bf16hi(u.y);
        q[4] = bf16lo(u.z); q[5] = bf16hi(u.z); q[6] = bf16lo(u.w); q[7] = bf16hi(u.w);
    }
    const uint16_t *base = static_cast<const uint16_t *>(p.Kmean) + bh * p.M_cap * kHeadDim + 8 * e;
    float *out = p.scores + bh * p.score_stride;

    const int m_begin = blk * 64 * p.iters + wave * 16;
    const int m_end = min((blk + 1) * 64 * p.iters, p.n_all);
    int left = (m_end - m_begin + 63) / 64;  // 16-row steps of this wave

    auto load = [&](int m0, uint4(&v)[4]) {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr)
            v[rr] = ld16_stream(base + (int64_t)min(m0 + 4 * rr + w, last_row) * kHeadDim);
    };
    auto finish = [&](int m0, const uint4(&v)[4]) {
        float mine = 0.f;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            float a = fmaf(q[0], bf16lo(v[rr].x), 0.f);  // from +0, so that a zero score is +0 (never -0) as in the fp32 kernel
            a = fmaf(q[1], bf16hi(v[rr].x), a);
            a = fmaf(q[2], bf16lo(v[rr].y), a);
            a = fmaf(q[3], bf16hi(v[rr].y), a);
            a = fmaf(q[4], bf16lo(v[rr].z), a);
            a = fmaf(q[5], bf16hi(v[rr].z), a);
            a = fmaf(q[6], bf16lo(v[rr].w), a);
            a = fmaf(q[7], bf16hi(v[rr].w), a);
            a += __shfl_xor(a, 1, kWave);
            a += __shfl_xor(a, 2, kWave);
            a += __shfl_xor(a, 4, kWave);
            a += __shfl_xor(a, 8, kWave);
            if (e == rr) mine = a;
        }
        // lane e < 4 stores row m0 + 4e + w
        const int m = m0 + 4 * e + w;
        if (e < 4 && m < p.n_all) __builtin_nontemporal_store(m < n ? mine : -INFINITY, &out[m]);
    };

    if (left > 0) {
        uint4 va[4], vb[4];
        int m0 = m_begin;
        load(m0, va);
        while (left > 2) {
            load(m0 + 64, vb);
            finish(m0, va);
            load(m0 + 128, va);
            finish(m0 + 64, vb);
            m0 += 128;
            left -= 2;
        }
        if (left == 2) {
            load(m0 + 64, vb);
            finish(m0, va);
            finish(m0 + 64, vb);
        } else {
            finish(m0, va);
        }
    }
}

// ascending order of keys == ascending order of the floats (-0 < +0, NaNs at the ends)
__device__ __forceinline__ uint32_t score_key(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// exclusive scan of one value per thread over a 1024-thread workgroup; *total = sum of all
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t *wave_tot /*[16]*/, uint32_t *total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t u = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += u;
    }
    __syncthreads();  // wave_tot may still be read from a previous scan
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kSelThreads / 64; ++w) {
        const uint32_t t = wave_tot[w];
        if (w < wave) before += t;
        all += t;
    }
    *total = all;
    return before + incl - v;
}

// kKeep > 0: a thread holds the keys of its contiguous index range [tid*per, tid*per+per),
// per <= kKeep, in registers -- the scores are read from memory once, and the four radix passes
// and the compaction run out of the register file (16 or 32 keys; 64 would spill at 1024 threads).
// kKeep == 0 (over 32768 chunks per head): every pass streams the scores again.
template <int kKeep>
__global__ __launch_bounds__(kSelThreads) void topk_select_kernel(const float *__restrict__ scores,
                                                                  int64_t score_stride,
                                                                  const int32_t *__restrict__ n_chunks, int n_all,
                                                                  int H, int k, int32_t *__restrict__ out_idx,
                                                                  float *__restrict__ out_score) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wtot[16];
    __shared__ uint32_t s_digit, s_remaining;
    __shared__ unsigned long long cand[TF_MAX_K_CHUNKS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t bh = blockIdx.x;
    const int b = (int)(bh / H);
    int n = n_chunks ? n_chunks[b] : n_all;
    n = min(max(n, 0), n_all);
    const int k_eff = min(k, n);
    const float *sc = scores + bh * score_stride;

    // thread t owns the contiguous index range [i_lo, i_hi); per is a multiple of 4 and the score
    // rows are padded to one, so the range is read as whole float4
    int per = (n + kSelThreads - 1) / kSelThreads;
    per = (per + 3) & ~3;
    const int i_lo = min(tid * per, n), i_hi = min(n, i_lo + per);

    uint32_t keys[kKeep > 0 ? kKeep : 1];
    if constexpr (kKeep > 0) {
#pragma unroll
        for (int u = 0; u < kKeep; u += 4) {
            float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k_eff > 0 && i_lo + u < i_hi) f = *reinterpret_cast<const float4 *>(sc + i_lo + u);
            keys[u] = score_key(f.x);
            keys[u + 1] = score_key(f.y);
            keys[u + 2] = score_key(f.z);
            keys[u + 3] = score_key(f.w);
        }
    }
    // f(key, index) for every key of this thread's range, in increasing index order
    auto for_owned = [&](auto &&f) {
        if constexpr (kKeep > 0) {
#pragma unroll
            for (int u = 0; u < kKeep; ++u)
                if (i_lo + u < i_hi) f(keys[u], i_lo + u);
        } else {
            for (int i = i_lo; i < i_hi; i += 4) {
                const float4 v = *reinterpret_cast<const float4 *>(sc + i);
                const float fv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (i + u < i_hi) f(score_key(fv[u]), i + u);
            }
        }
    };

    // ---- radix select: key of the k_eff-th largest score -------------------------------
    uint32_t prefix = 0, mask = 0, remaining = (uint32_t)k_eff;
    if (k_eff > 0) {
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            if constexpr (kKeep > 0) {
                for_owned([&](uint32_t key, int) {
                    if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
                });
            } else {
                for (int i = tid; i < n; i += kSelThreads) {  // order does not matter here: coalesced
                    const uint32_t key = score_key(sc[i]);
                    if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
                }
            }
            __syncthreads();
            // waves 0..3: suffix sums over the 256 bins (bin = tid)
            uint32_t hv = 0, incl = 0;
            if (tid < 256) {
                hv = hist[tid];
                incl = hv;
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    const uint32_t u = __shfl_down(incl, off, kWave);
                    if (lane + off < 64) incl += u;
                }
                if (lane == 0) wtot[wave] = incl;
            }
            __syncthreads();
            if (tid < 256) {
                uint32_t above = 0;  // elements in the bins of higher waves
                for (int w = wave + 1; w < 4; ++w) above += wtot[w];
                const uint32_t sfx = incl + above;   // elements in bins >= tid
                const uint32_t sfx_excl = sfx - hv;  // elements in bins  > tid
                if (sfx >= remaining && sfx_excl < remaining) {
                    s_digit = (uint32_t)tid;
                    s_remaining = remaining - sfx_excl;
                }
            }
            __syncthreads();
            prefix |= s_digit << shift;
            mask |= 0xffu << shift;
            remaining = s_remaining;
            __syncthreads();
        }
    }
    const uint32_t T = prefix;                        // key of the k_eff-th largest
    const uint32_t n_gt = (uint32_t)k_eff - remaining;  // keys strictly above T (all kept)

    // ---- ordered compaction of the winners (ties toward the lower index) ------------------
    uint32_t c_gt = 0, c_eq = 0;
    if (k_eff > 0)
        for_owned([&](uint32_t key, int) {
            c_gt += key > T;
            c_eq += key == T;
        });
    uint32_t tot_gt, tot_eq;
    uint32_t p_gt = block_excl_scan(c_gt, wtot, &tot_gt);
    uint32_t p_eq = block_excl_scan(c_eq, wtot, &tot_eq);
    if (k_eff > 0)
        for_owned([&](uint32_t key, int i) {
            const unsigned long long comp =
                ((unsigned long long)key << 32) | (unsigned long long)(0xffffffffu - (uint32_t)i);
            if (key > T) {
                cand[p_gt++] = comp;
            } else if (key == T) {
                if (p_eq < remaining) cand[n_gt + p_eq] = comp;
                ++p_eq;
            }
        });
    __syncthreads();

    // ---- order the winners: descending on (key, ~index) -----------------------------------
    // The composite values are distinct, so the place of a winner is the number of winners above
    // it. Counting that directly -- every thread walks the whole list, all lanes reading the same
    // LDS word per turn (a broadcast) -- takes k_eff turns without a barrier, against the
    // log^2(k) barrier-separated stages of a sorting network (45 stages for 512 winners).
    for (int j = tid; j < k_eff; j += kSelThreads) {
        const unsigned long long mine = cand[j];
        int above = 0;
#pragma unroll 8
        for (int i = 0; i < k_eff; ++i) above += cand[i] > mine;
        const int32_t idx = (int32_t)(0xffffffffu - (uint32_t)(mine & 0xffffffffull));
        out_idx[bh * k + above] = idx;
        if (out_score) out_score[bh * k + above] = sc[idx];
    }
    for (int j = k_eff + tid; j < k; j += kSelThreads) {  // fewer chunks than k: the rest is empty
        out_idx[bh * k + j] = -1;
        if (out_score) out_score[bh * k + j] = -INFINITY;
    }
}

// ---- fused scoring + selection ------------------------------------------------------------------
// One 512-thread workgroup per (b,h) streams that unit's average keys (the same loads and the same
// fp32 arithmetic as the scoring kernels above, so the scores are bit-equal to theirs), keeps the
// order-preserving keys of all scores in LDS and runs the radix select on them: the scores never
// travel to HBM and back, and while one workgroup of a compute unit selects, the other one streams.
// Used when there are enough units to fill the chip that way (see topk_gather_launch) and a unit's
// keys fit the LDS: up to kFusedMaxChunks chunks, 4 bytes each, plus 8 bytes per kept chunk.
constexpr int kFusedThreads = 512;
constexpr int kFusedMaxChunks = 16384;

// LDS position of chunk i's key: one word of padding per 32, so that threads reading contiguous
// ranges of 4..32 keys each spread over the banks
__device__ __forceinline__ int key_slot(int i) { return i + (i >> 5); }
static size_t fused_lds_bytes(int64_t n_all, int k) {
    const size_t words = (size_t)n_all + (size_t)(n_all >> 5) + 2;                // keys, padded; even count
    return ((words + 1) & ~(size_t)1) * 4 + (size_t)k * 8;                        // then the winners (8-byte aligned)
}

__device__ __forceinline__ float key_score(uint32_t key) {  // inverse of score_key
    return __uint_as_float((key & 0x80000000u) ? (key ^ 0x80000000u) : ~key);
}

struct FusedParams {
    const uint16_t *q_r;
    const void *Kmean;
    int64_t M_cap;
    const int32_t *n_chunks;
    int32_t n_all, H, k;
    int32_t *out_idx;
    float *out_score;
};

template <bool kBf16>
__global__ __launch_bounds__(kFusedThreads) void score_select_kernel(const FusedParams p) {
    extern __shared__ uint32_t sm_dyn[];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wtot[kFusedThreads / 64];
    __shared__ uint32_t s_digit, s_remaining;
    uint32_t *sm_key = sm_dyn;
    const int key_words = (p.n_all + (p.n_all >> 5) + 2 + 1) & ~1;
    unsigned long long *cand = reinterpret_cast<unsigned long long *>(sm_dyn + key_words);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int kWavesF = kFusedThreads / 64;
    const int64_t bh = blockIdx.x;
    const int b = (int)(bh / p.H);
    int n = p.n_chunks ? p.n_chunks[b] : p.n_all;
    n = min(max(n, 0), p.n_all);
    const int last_row = max(n - 1, 0);
    const int k = p.k, k_eff = min(k, n);

    // ---- phase 1: stream the table, one key per chunk into LDS ------------------------------
    // (rows past the sequence's chunk count are clamped to its last row: read, scored, never used)
    const int steps = (n + 15) / 16;                                   // 16-row steps of this unit
    if constexpr (!kBf16) {
        const int e = lane & 7, w = lane >> 3;
        float q[4][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint2 u = *reinterpret_cast<const uint2 *>(p.q_r + bh * kHeadDim + 32 * j + 4 * e);
            q[j][0] = bf16lo(u.x); q[j][1] = bf16hi(u.x); q[j][2] = bf16lo(u.y); q[j][3] = bf16hi(u.y);
        }
        const float *base = static_cast<const float *>(p.Kmean) + bh * p.M_cap * kHeadDim + 4 * e;
        auto load = [&](int m0, float4(&v)[8]) {
#pragma unroll
            for (int rr = 0; rr < 2; ++rr) {
                const float *row = base + (int64_t)min(m0 + 8 * rr + w, last_row) * kHeadDim;
#pragma unroll
                for (int j = 0; j < 4; ++j) v[4 * rr + j] = ldf4_stream(row + 32 * j);
            }
        };
        auto finish = [&](int m0, const float4(&v)[8]) {
            float acc[2];
#pragma unroll
            for (int rr = 0; rr < 2; ++rr) {
                float a = 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    a = fmaf(q[j][0], v[4 * rr + j].x, a);
                    a = fmaf(q[j][1], v[4 * rr + j].y, a);
                    a = fmaf(q[j][2], v[4 * rr + j].z, a);
                    a = fmaf(q[j][3], v[4 * rr + j].w, a);
                }
                a += __shfl_xor(a, 1, kWave);
                a += __shfl_xor(a, 2, kWave);
                a += __shfl_xor(a, 4, kWave);
                acc[rr] = a;
            }
            const int m = m0 + 8 * e + w;                               // lanes e = 0 / 1 keep rows m0 + w / m0 + 8 + w
            if (e < 2 && m < n) sm_key[key_slot(m)] = score_key(e == 0 ? acc[0] : acc[1]);
        };
        float4 va[8], vb[8];
        int i = wave;                                                   // the waves interleave 16-row steps
        if (i < steps) load(16 * i, va);
        for (; i + 2 * kWavesF < steps; i += 2 * kWavesF) {
            load(16 * (i + kWavesF), vb);
            finish(16 * i, va);
            load(16 * (i + 2 * kWavesF), va);
            finish(16 * (i + kWavesF), vb);
        }
        if (i + kWavesF < steps) {
            load(16 * (i + kWavesF), vb);
            finish(16 * i, va);
            finish(16 * (i + kWavesF), vb);
        } else if (i < steps) {
            finish(16 * i, va);
        }
    } else {
        const int e = lane & 15, w = lane >> 4;
        float q[8];
        {
            const uint4 u = ld16(p.q_r + bh * kHeadDim + 8 * e);
            q[0] = bf16lo(u.x); q[1] = bf16hi(u.x); q[2] = bf16lo(u.y); q[3] = bf16hi(u.y);
            q[4] = bf16lo(u.z); q[5] = bf16hi(u.z); q[6] = bf16lo(u.w); q[7] = bf16hi(u.w);
        }
        const uint16_t *base = static_cast<const uint16_t *>(p.Kmean) + bh * p.M_cap * kHeadDim + 8 * e;
        auto load = [&](int m0, uint4(&v)[4]) {
#pragma unroll
            for (int rr = 0; rr < 4; ++rr)
                v[rr] = ld16_stream(base + (int64_t)min(m0 + 4 * rr + w, last_row) * kHeadDim);
        };
        auto finish = [&](int m0, const uint4(&v)[4]) {
            float mine = 0.f;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                float a = fmaf(q[0], bf16lo(v[rr].x), 0.f);
                a = fmaf(q[1], bf16hi(v[rr].x), a);
                a = fmaf(q[2], bf16lo(v[rr].y), a);
                a = fmaf(q[3], bf16hi(v[rr].y), a);
                a = fmaf(q[4], bf16lo(v[rr].z), a);
                a = fmaf(q[5], bf16hi(v[rr].z), a);
                a = fmaf(q[6], bf16lo(v[rr].w), a);
                a = fmaf(q[7], bf16hi(v[rr].w), a);
                a += __shfl_xor(a, 1, kWave);
                a += __shfl_xor(a, 2, kWave);
                a += __shfl_xor(a, 4, kWave);
                a += __shfl_xor(a, 8, kWave);
                if (e == rr) mine = a;
            }
            const int m = m0 + 4 * e + w;                               // lane e < 4 keeps row m0 + 4e + w
            if (e < 4 && m < n) sm_key[key_slot(m)] = score_key(mine);
        };
        uint4 va[4], vb[4];
        int i = wave;
        if (i < steps) load(16 * i, va);
        for (; i + 2 * kWavesF < steps; i += 2 * kWavesF) {
            load(16 * (i + kWavesF), vb);
            finish(16 * i, va);
            load(16 * (i + 2 * kWavesF), va);
            finish(16 * (i + kWavesF), vb);
        }
        if (i + kWavesF < steps) {
            load(16 * (i + kWavesF), vb);
            finish(16 * i, va);
            finish(16 * (i + kWavesF), vb);
        } else if (i < steps) {
            finish(16 * i, va);
        }
    }
    __syncthreads();

    // ---- phase 2: radix select of the k_eff-th largest key (keys read from LDS) --------------
    uint32_t prefix = 0, mask = 0, remaining = (uint32_t)k_eff;
    if (k_eff > 0) {
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            for (int i = tid; i < n; i += kFusedThreads) {              // order does not matter here
                const uint32_t key = sm_key[key_slot(i)];
                if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
            }
            __syncthreads();
            uint32_t hv = 0, incl = 0;
            if (tid < 256) {                                            // waves 0..3: suffix sums over the bins
                hv = hist[tid];
                incl = hv;
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    const uint32_t u = __shfl_down(incl, off, kWave);
                    if (lane + off < 64) incl += u;
                }
                if (lane == 0) wtot[wave] = incl;
            }
            __syncthreads();
            if (tid < 256) {
                uint32_t above = 0;
                for (int w = wave + 1; w < 4; ++w) above += wtot[w];
                const uint32_t sfx = incl + above, sfx_excl = sfx - hv;
                if (sfx >= remaining && sfx_excl < remaining) {
                    s_digit = (uint32_t)tid;
                    s_remaining = remaining - sfx_excl;
                }
            }
            __syncthreads();
            prefix |= s_digit << shift;
            mask |= 0xffu << shift;
            remaining = s_remaining;
            __syncthreads();
        }
    }
    const uint32_t T = prefix;                          // key of the k_eff-th largest
    const uint32_t n_gt = (uint32_t)k_eff - remaining;  // keys strictly above T (all kept)

    // ---- ordered compaction: thread t owns the contiguous index range [i_lo, i_hi) -------------
    int per = (n + kFusedThreads - 1) / kFusedThreads;
    per = (per + 3) & ~3;
    const int i_lo = min(tid * per, n), i_hi = min(n, i_lo + per);
    uint32_t c_gt = 0, c_eq = 0;
    for (int i = i_lo; i < i_hi; ++i) {
        const uint32_t key = sm_key[key_slot(i)];
        c_gt += key > T;
        c_eq += key == T;
    }
    auto excl_scan = [&](uint32_t v, uint32_t *total) -> uint32_t {
        uint32_t incl = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t u = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += u;
        }
        __syncthreads();  // wtot may still be read from the previous use
        if (lane == 63) wtot[wave] = incl;
        __syncthreads();
        uint32_t before = 0, all = 0;
#pragma unroll
        for (int w = 0; w < kWavesF; ++w) {
            const uint32_t t = wtot[w];
            if (w < wave) before += t;
            all += t;
        }
        *total = all;
        return before + incl - v;
    };
    uint32_t tot_gt, tot_eq;
    uint32_t p_gt = excl_scan(c_gt, &tot_gt);
    uint32_t p_eq = excl_scan(c_eq, &tot_eq);
    if (k_eff > 0)
        for (int i = i_lo; i < i_hi; ++i) {
            const uint32_t key = sm_key[key_slot(i)];
            const unsigned long long comp =
                ((unsigned long long)key << 32) | (unsigned long long)(0xffffffffu - (uint32_t)i);
            if (key > T) {
                cand[p_gt++] = comp;
            } else if (key == T) {
                if (p_eq < remaining) cand[n_gt + p_eq] = comp;
                ++p_eq;
            }
        }
    __syncthreads();

    // ---- place of every winner on (key desc, index asc): the number of winners above it ----------
    for (int j = tid; j < k_eff; j += kFusedThreads) {
        const unsigned long long mine = cand[j];
        int above = 0;
#pragma unroll 8
        for (int i = 0; i < k_eff; ++i) above += cand[i] > mine;
        p.out_idx[bh * k + above] = (int32_t)(0xffffffffu - (uint32_t)(mine & 0xffffffffull));
        if (p.out_score) p.out_score[bh * k + above] = key_score((uint32_t)(mine >> 32));
    }
    for (int j = k_eff + tid; j < k; j += kFusedThreads) {  // fewer chunks than k: the rest is empty
        p.out_idx[bh * k + j] = -1;
        if (p.out_score) p.out_score[bh * k + j] = -INFINITY;
    }
}

struct GatherParams {
    const uint16_t *K, *V;
    uint16_t *Kr, *Vr;
    int64_t sb, sh, st;     // source strides
    int64_t rb, rh, rt;     // retrieval-cache strides
    const int32_t *idx;
    int32_t H, k, chunk, jblocks;
};

// A wave copies kCpw selected chunks: their indices first, then, four rows at a time, the rows of all
// of them are requested before the first is stored (2 kCpw loads of 16 bytes in flight per lane).
template <int kCpw>
__global__ __launch_bounds__(256) void chunk_gather_kernel(const GatherParams p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j0 = ((blockIdx.x % p.jblocks) * 4 + wave) * kCpw;
    const int64_t bh = blockIdx.x / p.jblocks;
    if (j0 >= p.k) return;
    int m[kCpw];
#pragma unroll
    for (int u = 0; u < kCpw; ++u) m[u] = j0 + u < p.k ? p.idx[bh * p.k + j0 + u] : -1;
    const int b = (int)(bh / p.H), h = (int)(bh - (int64_t)b * p.H);
    const int64_t src0 = (int64_t)b * p.sb + (int64_t)h * p.sh + (lane & 15) * 8;
    const int64_t dst0 = (int64_t)b * p.rb + (int64_t)h * p.rh + (int64_t)j0 * p.chunk * p.rt + (lane & 15) * 8;
    for (int i = lane >> 4; i < p.chunk; i += 4) {
        uint4 kv[kCpw], vv[kCpw];
#pragma unroll
        for (int u = 0; u < kCpw; ++u)
            if (m[u] >= 0) {
                const int64_t src = src0 + ((int64_t)m[u] * p.chunk + i) * p.st;
                kv[u] = ld16_stream(p.K + src);
                vv[u] = ld16_stream(p.V + src);
            }
#pragma unroll
        for (int u = 0; u < kCpw; ++u)
            if (m[u] >= 0) {
                const int64_t dst = dst0 + ((int64_t)u * p.chunk + i) * p.rt;
                st16_stream(p.Kr + dst, kv[u]);  // nt stores: 6% faster than plain ones here
                st16_stream(p.Vr + dst, vv[u]);
            }
    }
}

static int64_t score_stride_of(int64_t n_all) { return (n_all + 3) & ~(int64_t)3; }

size_t topk_workspace_bytes(int32_t batch, int32_t heads, int64_t n_chunks_all, int32_t k_chunks) {
    if (batch <= 0 || heads <= 0 || n_chunks_all <= 0 || k_chunks <= 0) return 0;
    // scores [BH][stride] fp32 (+ one float4 of slack for the vector loads of the last row)
    return ((size_t)batch * heads * score_stride_of(n_chunks_all) + 4) * sizeof(float);
}

int topk_gather_launch(const void *q_r, const void *Kmean, int64_t M_cap, const void *K, const void *V,
                       const tf_kv_desc *kd, int32_t chunk, const int32_t *n_chunks, int64_t n_chunks_all,
                       int32_t k_chunks, int32_t *out_idx, float *out_score, void *Kr, void *Vr,
                       const tf_kv_desc *rd, void *ws, size_t ws_bytes, void *stream, bool mean_bf16) {
    if (!q_r || !Kmean || !out_idx) return TF_ERR_INVALID_ARG;
    int rc = check_desc(kd);
    if (rc != TF_OK) return rc;
    const bool do_gather = Kr != nullptr || Vr != nullptr;
    if (do_gather) {
        if (!Kr || !Vr || !K || !V) return TF_ERR_INVALID_ARG;
        rc = check_desc(rd);
        if (rc != TF_OK) return rc;
        if (rd->batch != kd->batch || rd->heads != kd->heads) return TF_ERR_INVALID_ARG;
        if ((int64_t)k_chunks * chunk > rd->capacity) return TF_ERR_INVALID_ARG;
        if (!aligned(K, 16) || !aligned(V, 16) || !aligned(Kr, 16) || !aligned(Vr, 16)) return TF_ERR_INVALID_ARG;
    }
    if (chunk < 1 || k_chunks < 1 || n_chunks_all < 1 || M_cap < 1) return TF_ERR_INVALID_ARG;
    if (chunk > 64 || k_chunks > TF_MAX_K_CHUNKS) return TF_ERR_UNSUPPORTED;
    if (n_chunks_all > M_cap || k_chunks > n_chunks_all) return TF_ERR_INVALID_ARG;
    if (n_chunks_all > ((int64_t)1 << 30)) return TF_ERR_UNSUPPORTED;
    if (n_chunks_all * chunk > kd->capacity) return TF_ERR_INVALID_ARG;
    if (!aligned(q_r, mean_bf16 ? 16 : 8) || !aligned(Kmean, 16)) return TF_ERR_INVALID_ARG;
    if (!ws || !aligned(ws, 256) ||
        ws_bytes < topk_workspace_bytes(kd->batch, kd->heads, n_chunks_all, k_chunks))
        return TF_ERR_WORKSPACE;

    const int64_t BH = (int64_t)kd->batch * kd->heads;
    hipStream_t st = static_cast<hipStream_t>(stream);

    // Fused scoring + selection when a unit's keys fit the LDS and there are at least two units per
    // compute unit (one streams while the other selects; with fewer units most of the chip would idle
    // and the three-kernel path, which spreads one unit over many workgroups, is faster).
    const int64_t fused_opt = fused_option();
    bool fused = fused_opt != 2 && n_chunks_all <= kFusedMaxChunks &&
                 (fused_opt == 1 || BH >= 2 * (int64_t)compute_units());
    if (fused) {
        const size_t lds = fused_lds_bytes(n_chunks_all, k_chunks);
        const void *fn = mean_bf16 ? reinterpret_cast<const void *>(&score_select_kernel<true>)
                                   : reinterpret_cast<const void *>(&score_select_kernel<false>);
        // more than 64 KiB of dynamic LDS has to be allowed per kernel; if the runtime refuses, the
        // three-kernel path below serves the call
        if (lds > (size_t)64 << 10 &&
            hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            fused = false;
        }
        if (fused) {
            FusedParams fp;
            fp.q_r = static_cast<const uint16_t *>(q_r);
            fp.Kmean = Kmean;
            fp.M_cap = M_cap;
            fp.n_chunks = n_chunks;
            fp.n_all = (int32_t)n_chunks_all;
            fp.H = kd->heads;
            fp.k = k_chunks;
            fp.out_idx = out_idx;
            fp.out_score = out_score;
            if (mean_bf16)
                hipLaunchKernelGGL(score_select_kernel<true>, dim3((unsigned)BH), dim3(kFusedThreads), lds, st, fp);
            else
                hipLaunchKernelGGL(score_select_kernel<false>, dim3((unsigned)BH), dim3(kFusedThreads), lds, st, fp);
        }
    }

    ScoreParams sp;
    sp.q_r = static_cast<const uint16_t *>(q_r);
    sp.Kmean = Kmean;
    sp.M_cap = M_cap;
    sp.n_chunks = n_chunks;
    sp.n_all = (int32_t)n_chunks_all;
    sp.H = kd->heads;
    // steps per wave: long tables give every workgroup up to 1024 rows (512 KiB), short ones
    // keep at least ~2048 workgroups in the launch
    int64_t iters = n_chunks_all * BH / (64 * 2048);
    iters = iters < 1 ? 1 : (iters > kScoreMaxIters ? kScoreMaxIters : iters);
    if (const int64_t forced = score_iters_option(); forced > 0) iters = forced;
    sp.iters = (int32_t)iters;
    sp.blocks_per_bh = (int32_t)((n_chunks_all + 64 * iters - 1) / (64 * iters));
    sp.scores = static_cast<float *>(ws);
    sp.score_stride = score_stride_of(n_chunks_all);
    if (sp.blocks_per_bh * BH >= (int64_t)1 << 31) return TF_ERR_UNSUPPORTED;
    if (!fused) {
        if (mean_bf16)
            hipLaunchKernelGGL(chunk_score_bf16_kernel, dim3((unsigned)(sp.blocks_per_bh * BH)), dim3(256), 0, st, sp);
        else
            hipLaunchKernelGGL(chunk_score_kernel, dim3((unsigned)(sp.blocks_per_bh * BH)), dim3(256), 0, st, sp);
    }

    auto select = [&](auto keep_tag) {
        hipLaunchKernelGGL((topk_select_kernel<decltype(keep_tag)::value>), dim3((unsigned)BH), dim3(kSelThreads), 0,
                           st, sp.scores, sp.score_stride, n_chunks, (int)n_chunks_all, (int)kd->heads,
                           (int)k_chunks, out_idx, out_score);
    };
    if (fused) {
        // idx and scores are already on their way
    } else if (n_chunks_all <= 16 * kSelThreads) select(std::integral_constant<int, 16>{});
    else if (n_chunks_all <= 32 * kSelThreads) select(std::integral_constant<int, 32>{});
    else select(std::integral_constant<int, 0>{});

    if (do_gather) {
        GatherParams gp;
        gp.K = static_cast<const uint16_t *>(K);
        gp.V = static_cast<const uint16_t *>(V);
        gp.Kr = static_cast<uint16_t *>(Kr);
        gp.Vr = static_cast<uint16_t *>(Vr);
        gp.sb = kd->stride_b;
        gp.sh = kd->stride_h;
        gp.st = kd->stride_t;
        gp.rb = rd->stride_b;
        gp.rh = rd->stride_h;
        gp.rt = rd->stride_t;
        gp.idx = out_idx;
        gp.H = kd->heads;
        gp.k = k_chunks;
        gp.chunk = chunk;
        // chunks per wave, measured on the 32-layer rebuild (4 GiB read + written): 1: 5.8-5.9 TB/s, 2: 5.7-5.9,
        // 4: 5.5, 8: 5.6 -- the copy is bound by the mixed read/write rate of the memory, not by loads in flight
        constexpr int kCpw = 1;
        gp.jblocks = (k_chunks + 4 * kCpw - 1) / (4 * kCpw);
        hipLaunchKernelGGL(chunk_gather_kernel<kCpw>, dim3((unsigned)(gp.jblocks * BH)), dim3(256), 0, st, gp);
    }
    return hip_status(hipGetLastError());
}

}  // namespace tf
