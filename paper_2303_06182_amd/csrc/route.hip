// Routing kernels: softmax + top-k over the gate logits, per-expert counts with a prefix
// scan, the stable permutation of the assignments, and the M-tile map of the grouped GEMM.
//
// Paper: top-1 / top-2 gating (Sec. 2.3); dynamic gating sorts the expert assignments and counts
// the occurrences of each expert (Sec. 5.1).  The sort here is a counting sort: its result is the
// stable argsort (ascending token inside each expert) and costs O(N) instead of O(N log N).
// Nothing uses atomics on global memory, so the permutation is the same on every run.
#include "moe_internal.h"

namespace moe355 {

static constexpr int kThreads = 256;
static constexpr int kWave = 64;
static constexpr int kMaxLogitParts = 16;  // slices the top-k kernel can add up (the gate GEMM's split K)

// ------------------------------------------------------------------------------------------------
// softmax + top-k.  G lanes (a power of two <= 64) share one token; lane `sub` holds logits
// sub, sub+G, sub+2G, ...  Each of the k rounds takes the largest remaining logit; equal logits
// go to the lower expert index (inside a lane indices ascend with the register slot, across
// lanes the butterfly compares (value, index)).
// ------------------------------------------------------------------------------------------------
// VEC: lane `sub` instead holds the 16-byte groups sub, sub+G, ... of the row (4 logits each, E a
// multiple of 4), so every lane has V/4 float4 loads in flight; slot i of the lane is expert
// (i/4)*4G + 4*sub + i%4, still ascending with i.
template <int G, int V, bool VEC>
// n_parts > 1: the logits arrive as n_parts partial sums (the gate GEMM's split K): slice 0 at `logits`,
// slice i > 0 at parts + (i - 1) * part_stride; they are added in slice order and the sum is written
// back to `logits`.
__global__ __launch_bounds__(kThreads) void topk_kernel(float *logits, int T, int E, int k, int renorm,
                                                        int32_t *__restrict__ idx, float *__restrict__ w,
                                                        int n_parts, const float *__restrict__ parts,
                                                        int64_t part_stride)
{
    constexpr int TOK_PER_BLOCK = kThreads / G;
    const int sub = threadIdx.x % G;
    const int t = blockIdx.x * TOK_PER_BLOCK + threadIdx.x / G;
    const bool live = t < T;
    const float NEG_INF = -__builtin_huge_valf();
    auto expert_of = [&](int i) { return VEC ? (i >> 2) * (4 * G) + 4 * sub + (i & 3) : sub + i * G; };

    float v[V];
    if (VEC) {
#pragma unroll
        for (int q = 0; q < V / 4; ++q) {
            const int e0 = (q * G + sub) * 4;
            float4 f = make_float4(NEG_INF, NEG_INF, NEG_INF, NEG_INF);
            if (live && e0 < E) {
                float *src = logits + (int64_t)t * E + e0;
                f = *reinterpret_cast<const float4 *>(src);
                if (n_parts > 1) {  // uniform over the grid; all slices are requested before the first is added
                    float4 g[kMaxLogitParts - 1];
#pragma unroll
                    for (int sp = 1; sp < kMaxLogitParts; ++sp)
                        g[sp - 1] = sp < n_parts ? *reinterpret_cast<const float4 *>(parts + (sp - 1) * part_stride +
                                                                                     (int64_t)t * E + e0)
                                                 : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                    for (int sp = 1; sp < kMaxLogitParts; ++sp) {
                        if (sp < n_parts) {
                            f.x += g[sp - 1].x;
                            f.y += g[sp - 1].y;
                            f.z += g[sp - 1].z;
                            f.w += g[sp - 1].w;
                        }
                    }
                    *reinterpret_cast<float4 *>(src) = f;
                }
            }
            v[(4 * q + 0) % V] = f.x;
            v[(4 * q + 1) % V] = f.y;
            v[(4 * q + 2) % V] = f.z;
            v[(4 * q + 3) % V] = f.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const int e = sub + i * G;
            v[i] = NEG_INF;
            if (live && e < E) {
                float *src = logits + (int64_t)t * E + e;
                float f = *src;
                if (n_parts > 1) {
                    float g[kMaxLogitParts - 1];
#pragma unroll
                    for (int sp = 1; sp < kMaxLogitParts; ++sp)
                        g[sp - 1] = sp < n_parts ? parts[(sp - 1) * part_stride + (int64_t)t * E + e] : 0.f;
#pragma unroll
                    for (int sp = 1; sp < kMaxLogitParts; ++sp)
                        if (sp < n_parts) f += g[sp - 1];
                    *src = f;
                }
                v[i] = f;
            }
        }
    }
    uint32_t taken = 0;  // bit i: register slot i already selected (or beyond E)
#pragma unroll
    for (int i = 0; i < V; ++i)
        if (expert_of(i) >= E) taken |= 1u << i;

    float sel_v[MOE_MAX_K];
    int sel_e[MOE_MAX_K];
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j) {
        sel_v[j] = NEG_INF;
        sel_e[j] = 0;
        if (j >= k) continue;  // uniform over the block
        float bv = NEG_INF;
        int be = 0x7fffffff;  // "none"
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const bool free_slot = !((taken >> i) & 1u);
            if (free_slot && (be == 0x7fffffff || v[i] > bv)) {
                bv = v[i];
                be = expert_of(i);
            }
        }
#pragma unroll
        for (int off = G / 2; off >= 1; off >>= 1) {
            const float ov = __shfl_xor(bv, off, kWave);
            const int oe = __shfl_xor(be, off, kWave);
            const bool other_wins = (oe != 0x7fffffff) && (be == 0x7fffffff || ov > bv || (ov == bv && oe < be));
            if (other_wins) {
                bv = ov;
                be = oe;
            }
        }
        // every lane of the group agrees for finite inputs; take lane 0's view so that the
        // "taken" bookkeeping stays consistent whatever the inputs are
        const int base = (threadIdx.x % kWave) - sub;
        bv = __shfl(bv, base, kWave);
        be = __shfl(be, base, kWave);
        sel_v[j] = bv;
        sel_e[j] = be;
        if (be != 0x7fffffff) {
            const int owner = VEC ? (be % (4 * G)) >> 2 : be % G;
            const int slot = VEC ? (be / (4 * G)) * 4 + (be & 3) : be / G;
            if (owner == sub) taken |= 1u << slot;
        }
    }

    // gate weights in fp32: exp(l - max) over the selected (renorm) or over all experts
    const float m = sel_v[0];
    float denom = 0.f;
    if (renorm) {
#pragma unroll
        for (int j = 0; j < MOE_MAX_K; ++j)
            if (j < k) denom += expf(sel_v[j] - m);
    } else {
        float part = 0.f;
#pragma unroll
        for (int i = 0; i < V; ++i)
            if (expert_of(i) < E) part += expf(v[i] - m);
#pragma unroll
        for (int off = G / 2; off >= 1; off >>= 1) part += __shfl_xor(part, off, kWave);
        denom = part;
    }
    if (live && sub == 0) {
#pragma unroll
        for (int j = 0; j < MOE_MAX_K; ++j) {
            if (j < k) {
                idx[(int64_t)t * k + j] = sel_e[j];
                w[(int64_t)t * k + j] = expf(sel_v[j] - m) / denom;
            }
        }
    }
}

template <int G, int V, bool VEC>
static int launch_topk_t(float *logits, int T, int E, int k, int renorm, int32_t *idx, float *w, hipStream_t s,
                         int n_parts, const float *parts, int64_t part_stride)
{
    const int tpb = kThreads / G;
    ProfScope ps("topk", s);
    hipLaunchKernelGGL((topk_kernel<G, V, VEC>), dim3(ceil_div(T, tpb)), dim3(kThreads), 0, s, logits, T, E, k, renorm,
                       idx, w, n_parts, parts, part_stride);
    MOE_LAUNCH_CHECK("topk_kernel");
    return MOE_OK;
}

int launch_topk(float *logits, int T, int E, int k, int renorm, int32_t *idx, float *w, hipStream_t s, int n_parts,
                const float *parts, int64_t part_stride)
{
    if (T == 0) return MOE_OK;
    if (n_parts > kMaxLogitParts) {
        set_error("top-k: %d logit slices, at most %d", n_parts, kMaxLogitParts);
        return MOE_ERR_INVALID_ARG;
    }
    if (E % 4 == 0) {  // rows are 16-byte aligned: vector loads, fewer lanes per token
        if (E <= 8) return launch_topk_t<2, 4, true>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
        if (E <= 16) return launch_topk_t<4, 4, true>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
        if (E <= 32) return launch_topk_t<8, 4, true>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
        if (E <= 64) return launch_topk_t<16, 4, true>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
        if (E <= 128) return launch_topk_t<16, 8, true>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
        if (E <= 256) return launch_topk_t<16, 16, true>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
        if (E <= 512) return launch_topk_t<32, 16, true>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
        return launch_topk_t<64, 16, true>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
    }
    if (E <= 4) return launch_topk_t<4, 1, false>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
    if (E <= 8) return launch_topk_t<8, 1, false>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
    if (E <= 16) return launch_topk_t<16, 1, false>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
    if (E <= 32) return launch_topk_t<32, 1, false>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
    if (E <= 64) return launch_topk_t<64, 1, false>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
    if (E <= 128) return launch_topk_t<64, 2, false>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
    if (E <= 256) return launch_topk_t<64, 4, false>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
    if (E <= 512) return launch_topk_t<64, 8, false>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
    return launch_topk_t<64, 16, false>(logits, T, E, k, renorm, idx, w, s, n_parts, parts, part_stride);
}

// ------------------------------------------------------------------------------------------------
// counts / offsets / stable permutation.
//   K1 route_hist : block b histograms its 256 tokens into LDS -> block_hist[b][e]
//                   (the fused gate kernel writes these rows itself, one per tile of its own)
//   K2 route_prefix: per expert (one wave each), exclusive prefix over the rows (block_hist becomes
//                   the base of row b inside expert e) and counts[e]
//   K3 route_rank : every block scans the counts into offsets[] (wave-shuffle scan), then ranks its
//                   tokens: bit-wise ballots find equal experts inside a wave, an LDS prefix runs over
//                   the 4 waves, plus the row base and the expert offset
// ------------------------------------------------------------------------------------------------
int route_blocks(int T) { return T > 0 ? ceil_div(T, kThreads) : 1; }

__device__ __forceinline__ int clamp_expert(int e, int E) { return e < 0 ? 0 : (e >= E ? E - 1 : e); }

__global__ __launch_bounds__(kThreads) void route_hist_kernel(const int32_t *__restrict__ idx, int T, int E, int k,
                                                              int32_t *__restrict__ block_hist)
{
    __shared__ int hist[MOE_MAX_E];
    for (int e = threadIdx.x; e < E; e += kThreads) hist[e] = 0;
    __syncthreads();
    const int t = blockIdx.x * kThreads + threadIdx.x;
    if (t < T) {
        for (int j = 0; j < k; ++j) atomicAdd(&hist[clamp_expert(idx[(int64_t)t * k + j], E)], 1);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += kThreads) block_hist[(int64_t)blockIdx.x * E + e] = hist[e];
}

// Per expert, the exclusive prefix of its histogram column over the rows (blocks of tokens) and its total.
// One wave per expert, 64 rows per step: the column is walked with a wave-shuffle scan and a running carry.
// hist[b][e] becomes the number of assignments to expert e in the rows before b.
__global__ __launch_bounds__(kThreads) void route_prefix_kernel(int32_t *__restrict__ hist, int nrows, int E,
                                                                int32_t *__restrict__ counts)
{
    const int lane = threadIdx.x % kWave;
    const int e = blockIdx.x * (kThreads / kWave) + threadIdx.x / kWave;
    if (e >= E) return;  // whole waves leave together
    int carry = 0;
    for (int b0 = 0; b0 < nrows; b0 += kWave) {
        const int b = b0 + lane;
        const int v = b < nrows ? hist[(int64_t)b * E + e] : 0;
        int incl = v;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const int up = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += up;
        }
        if (b < nrows) hist[(int64_t)b * E + e] = carry + incl - v;
        carry += __shfl(incl, kWave - 1, kWave);
    }
    if (lane == 0) counts[e] = carry;
}

// Exclusive scan of n <= 4 * blockDim values in LDS (in place), one block; returns nothing, `total` receives
// the sum.  Thread t owns elements 4 t .. 4 t + 3.
__device__ __forceinline__ void block_exclusive_scan4(int *vals, int n, int *wave_tot, int &total)
{
    const int lane = threadIdx.x % kWave;
    const int wave = threadIdx.x / kWave;
    const int nw = blockDim.x / kWave;
    int loc[4];
    int sum = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int at = 4 * threadIdx.x + i;
        loc[i] = at < n ? vals[at] : 0;
        sum += loc[i];
    }
    int incl = sum;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int up = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += up;
    }
    if (lane == kWave - 1) wave_tot[wave] = incl;
    __syncthreads();
    int run = incl - sum;
    int all = 0;
    for (int w2 = 0; w2 < nw; ++w2) {
        const int t = wave_tot[w2];
        if (w2 < wave) run += t;
        all += t;
    }
    total = all;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int at = 4 * threadIdx.x + i;
        if (at < n) vals[at] = run;
        run += loc[i];
    }
    __syncthreads();
}

// Stable position of every assignment.  Block b ranks its 256 tokens:
//   row(t, j) = offsets[e] + (assignments to e in the blocks before b) + (in the waves before this one)
//               + (in the lanes before this one, or in earlier slots of this lane)
// Every block scans the E counts into the offsets itself (E <= 1024 integers out of L2), so no launch stands
// between the per-expert prefix and the ranking; block 0 also writes offsets[] and, when asked, the grouped
// GEMM's M-tile map.
// Equal experts inside a wave are found with one ballot per BIT of the expert index (ceil(log2 E) of them
// per slot) instead of one per expert: the lanes whose slot j' holds this lane's expert are the AND over the
// bits b of (bit b of my expert set ? ballot(bit b set) : its complement).
// hist_row_step: histogram rows per block of 256 tokens (the fused gate kernel's tiles may be shorter).
template <int KMAX>
__global__ __launch_bounds__(kThreads) void route_rank_kernel(const int32_t *__restrict__ idx, int T, int E, int k,
                                                              int nbits, const int32_t *__restrict__ counts,
                                                              const int32_t *__restrict__ block_base,
                                                              int hist_row_step, int32_t *__restrict__ offsets,
                                                              int32_t *__restrict__ dst_row,
                                                              int32_t *__restrict__ src_tok, int tile_bm,
                                                              int32_t *__restrict__ tile_expert,
                                                              int32_t *__restrict__ tile_row,
                                                              int32_t *__restrict__ num_tiles, int max_m_tiles)
{
    constexpr int NW = kThreads / kWave;
    __shared__ int offs[MOE_MAX_E];
    __shared__ int wave_cnt[NW][MOE_MAX_E];
    __shared__ int wave_tot[NW];
    const int lane = threadIdx.x % kWave;
    const int wave = threadIdx.x / kWave;
    const int t = blockIdx.x * kThreads + threadIdx.x;

    for (int e = threadIdx.x; e < E; e += kThreads) {
        offs[e] = counts[e];
#pragma unroll
        for (int w2 = 0; w2 < NW; ++w2) wave_cnt[w2][e] = 0;
    }
    __syncthreads();
    int total = 0;
    block_exclusive_scan4(offs, E, wave_tot, total);  // offs[e] = first row of expert e
    if (blockIdx.x == 0) {
        for (int e = threadIdx.x; e < E; e += kThreads) offsets[e] = offs[e];
        if (threadIdx.x == 0) offsets[E] = total;
    }

    int ej[KMAX];
    int below[KMAX];  // assignments to the same expert earlier in this wave
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
        ej[j] = (t < T && j < k) ? clamp_expert(idx[(int64_t)t * k + j], E) : -1;
        below[j] = 0;
    }
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (kWave - lane));
    const uint64_t gt_mask = (lane == kWave - 1) ? 0ull : (~0ull << (lane + 1));
    int after[KMAX];  // ... later in this wave
#pragma unroll
    for (int j = 0; j < KMAX; ++j) after[j] = 0;
#pragma unroll
    for (int jp = 0; jp < KMAX; ++jp) {
        if (jp >= k) continue;  // uniform
        uint64_t same[KMAX];
        const uint64_t valid = __ballot(ej[jp] >= 0);
#pragma unroll
        for (int j = 0; j < KMAX; ++j) same[j] = valid;
        for (int b = 0; b < nbits; ++b) {
            const uint64_t bal = __ballot(ej[jp] >= 0 && ((ej[jp] >> b) & 1));
#pragma unroll
            for (int j = 0; j < KMAX; ++j) same[j] &= ((ej[j] >> b) & 1) ? bal : ~bal;
        }
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
            if (ej[j] < 0) continue;
            below[j] += __popcll(same[j] & lt_mask);
            after[j] += __popcll(same[j] & gt_mask);
            // the lane's own other slots (only a caller's duplicate experts make these match)
            if (jp < j && ej[jp] == ej[j]) below[j] += 1;
            if (jp > j && ej[jp] == ej[j]) after[j] += 1;
        }
    }
    // the last assignment of every expert present in the wave publishes the wave's count of it
#pragma unroll
    for (int j = 0; j < KMAX; ++j)
        if (ej[j] >= 0 && after[j] == 0) wave_cnt[wave][ej[j]] = below[j] + 1;
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += kThreads) {
        int run = 0;
#pragma unroll
        for (int w2 = 0; w2 < NW; ++w2) {
            const int c = wave_cnt[w2][e];
            wave_cnt[w2][e] = run;
            run += c;
        }
    }
    __syncthreads();
    if (t < T) {
        const int32_t *base = block_base + (int64_t)blockIdx.x * hist_row_step * E;
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
            if (j < k) {
                const int e = ej[j];
                const int r = offs[e] + base[e] + wave_cnt[wave][e] + below[j];
                dst_row[(int64_t)t * k + j] = r;
                src_tok[r] = t;
            }
        }
    }
    if (tile_bm > 0 && blockIdx.x == 0) {  // the grouped GEMM's M-tile map: expert e owns ceil(count / tile_bm) tiles
        __syncthreads();
        int *first = &wave_cnt[0][0];  // reused: first tile of every expert
        for (int e = threadIdx.x; e < E; e += kThreads) first[e] = (counts[e] + tile_bm - 1) / tile_bm;
        __syncthreads();
        int n_tiles = 0;
        block_exclusive_scan4(first, E, wave_tot, n_tiles);
        for (int e = threadIdx.x; e < E; e += kThreads) {
            const int nt = (counts[e] + tile_bm - 1) / tile_bm;
            for (int i = 0; i < nt; ++i) {
                const int ti = first[e] + i;
                if (ti < max_m_tiles) {
                    tile_expert[ti] = e;
                    tile_row[ti] = offs[e] + i * tile_bm;
                }
            }
        }
        if (threadIdx.x == 0) num_tiles[0] = min(n_tiles, max_m_tiles);
    }
}

// ------------------------------------------------------------------------------------------------
// Small batches (decoder steps: a few hundred assignments): the three kernels above are then all
// launch latency, so one block of 1024 threads does the whole job in LDS -- histogram, scan,
// tile map and ranks -- with one thread per assignment a = t*k + j, in chunks of 1024.  The rank
// of a inside its expert is (assignments of that expert in earlier chunks and waves) + (lanes
// below it in its wave with the same expert); waves add their counts to the running per-expert
// totals one after the other, so the order is that of a, as in the kernels above.
// ------------------------------------------------------------------------------------------------
static constexpr int kSmallRouteMax = 4096;  // assignments

__global__ __launch_bounds__(1024) void route_small_kernel(const int32_t *__restrict__ idx, int n_assign, int E, int k,
                                                           int32_t *__restrict__ counts,
                                                           int32_t *__restrict__ offsets,
                                                           int32_t *__restrict__ dst_row,
                                                           int32_t *__restrict__ src_tok, int tile_bm,
                                                           int32_t *__restrict__ tile_expert,
                                                           int32_t *__restrict__ tile_row,
                                                           int32_t *__restrict__ num_tiles, int max_m_tiles)
{
    __shared__ int hist[MOE_MAX_E];   // counts, then the running totals of the ranking pass
    __shared__ int start[MOE_MAX_E];  // first row of every expert
    __shared__ int wave_tot[16];
    const int lane = threadIdx.x % kWave;
    const int wave = threadIdx.x / kWave;
    for (int e = threadIdx.x; e < MOE_MAX_E; e += 1024) hist[e] = 0;
    __syncthreads();
    for (int a = threadIdx.x; a < n_assign; a += 1024) atomicAdd(&hist[clamp_expert(idx[a], E)], 1);
    __syncthreads();
    // exclusive scan over the experts: thread e owns expert e (E <= 1024)
    const int cnt = threadIdx.x < E ? hist[threadIdx.x] : 0;
    int incl = cnt;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int up = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += up;
    }
    if (lane == kWave - 1) wave_tot[wave] = incl;
    __syncthreads();
    int wbase = 0;
    for (int w2 = 0; w2 < wave; ++w2) wbase += wave_tot[w2];
    const int my_off = wbase + incl - cnt;
    if (threadIdx.x < E) {
        counts[threadIdx.x] = cnt;
        offsets[threadIdx.x] = my_off;
        start[threadIdx.x] = my_off;
    }
    if (threadIdx.x == 0) offsets[E] = n_assign;
    if (tile_bm > 0) {  // uniform over the block: the grouped GEMM's M-tile map, as route_rank_kernel's block 0 writes it
        const int nt = (threadIdx.x < E && cnt > 0) ? (cnt + tile_bm - 1) / tile_bm : 0;
        int incl_t = nt;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const int up = __shfl_up(incl_t, off, kWave);
            if (lane >= off) incl_t += up;
        }
        __syncthreads();  // wave_tot is reused
        if (lane == kWave - 1) wave_tot[wave] = incl_t;
        __syncthreads();
        int tbase = 0;
        for (int w2 = 0; w2 < wave; ++w2) tbase += wave_tot[w2];
        const int first = tbase + incl_t - nt;
        for (int i = 0; i < nt; ++i) {
            const int ti = first + i;
            if (ti < max_m_tiles) {
                tile_expert[ti] = threadIdx.x;
                tile_row[ti] = my_off + i * tile_bm;
            }
        }
        if (threadIdx.x == 1023) num_tiles[0] = min(first + nt, max_m_tiles);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < MOE_MAX_E; e += 1024) hist[e] = 0;  // now: assignments ranked so far
    __syncthreads();
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (kWave - lane));
    for (int a0 = 0; a0 < n_assign; a0 += 1024) {  // trip count uniform over the block
        const int a = a0 + threadIdx.x;
        const bool live = a < n_assign;
        const int e = live ? clamp_expert(idx[a], E) : -1;
        // lanes of the wave with the same expert: one ballot per distinct expert present
        int below = 0, same = 0, leader = 0;
        uint64_t todo = __ballot(live);
        while (todo) {
            const int src = __ffsll((unsigned long long)todo) - 1;
            const int e0 = __shfl(e, src, kWave);
            const uint64_t mask = __ballot(e == e0);
            if (e == e0) {
                below = __popcll(mask & lt_mask);
                same = __popcll(mask);
                leader = (lane == src);
            }
            todo &= ~mask;
        }
        // the waves take their turns in order; the first lane of every expert group moves the total
        int base = 0;
        const int live_waves = min(16, (n_assign - a0 + kWave - 1) / kWave);  // uniform over the block
        for (int w2 = 0; w2 < live_waves; ++w2) {
            if (wave == w2 && live && leader) {
                base = hist[e];
                hist[e] = base + same;
            }
            __syncthreads();
        }
        // hand the group's base to its other lanes
        {
            uint64_t todo2 = __ballot(live);
            int got = base;
            while (todo2) {
                const int src = __ffsll((unsigned long long)todo2) - 1;
                const int e0 = __shfl(e, src, kWave);
                const int b0 = __shfl(base, src, kWave);
                const uint64_t mask = __ballot(e == e0);
                if (e == e0) got = b0;
                todo2 &= ~mask;
            }
            base = got;
        }
        if (live) {
            const int r = start[e] + base + below;
            dst_row[a] = r;
            src_tok[r] = a / k;
        }
    }
}

bool route_uses_hist(int T, int k) { return (int64_t)T * k > kSmallRouteMax; }

int launch_route(const int32_t *idx, int T, int E, int k, int32_t *counts, int32_t *offsets, int32_t *dst_row,
                 int32_t *src_tok, int32_t *block_hist, hipStream_t s, int tile_bm, int32_t *tile_expert,
                 int32_t *tile_row, int32_t *num_tiles, int max_m_tiles, int hist_tokens)
{
    ProfScope ps("route", s);  // histogram + prefix + rank together
    if ((int64_t)T * k <= kSmallRouteMax) {
        hipLaunchKernelGGL(route_small_kernel, dim3(1), dim3(1024), 0, s, idx, T * k, E, k, counts, offsets, dst_row,
                           src_tok, tile_bm, tile_expert, tile_row, num_tiles, max_m_tiles);
        MOE_LAUNCH_CHECK("route_small_kernel");
        return MOE_OK;
    }
    // hist_tokens > 0: block_hist already holds one histogram row per hist_tokens tokens (the fused gate kernel
    // wrote it); else it is made here, one row per block of 256 tokens
    if (hist_tokens > 0 && (kThreads % hist_tokens != 0)) {
        set_error("route: %d tokens per histogram row do not divide %d", hist_tokens, kThreads);
        return MOE_ERR_INVALID_ARG;
    }
    const int nblk = route_blocks(T);
    int nrows = nblk, row_step = 1;
    if (hist_tokens > 0) {
        nrows = ceil_div(T, hist_tokens);
        row_step = kThreads / hist_tokens;
    } else {
        hipLaunchKernelGGL(route_hist_kernel, dim3(nblk), dim3(kThreads), 0, s, idx, T, E, k, block_hist);
        MOE_LAUNCH_CHECK("route_hist_kernel");
    }
    hipLaunchKernelGGL(route_prefix_kernel, dim3(ceil_div(E, kThreads / kWave)), dim3(kThreads), 0, s, block_hist,
                       nrows, E, counts);
    MOE_LAUNCH_CHECK("route_prefix_kernel");
    int nbits = 0;
    while ((1 << nbits) < E) ++nbits;
#define MOE_RANK(KM)                                                                                              \
    hipLaunchKernelGGL(route_rank_kernel<KM>, dim3(nblk), dim3(kThreads), 0, s, idx, T, E, k, nbits, counts,      \
                       block_hist, row_step, offsets, dst_row, src_tok, tile_bm, tile_expert, tile_row, num_tiles, \
                       max_m_tiles)
    // KMAX = slots a lane holds: the smallest instantiation that holds k
    if (k <= 1) MOE_RANK(1);
    else if (k <= 2) MOE_RANK(2);
    else if (k <= 4) MOE_RANK(4);
    else MOE_RANK(MOE_MAX_K);
#undef MOE_RANK
    MOE_LAUNCH_CHECK("route_rank_kernel");
    return MOE_OK;
}

// ------------------------------------------------------------------------------------------------
// M-tile map of the grouped GEMM: expert e owns ceil(count_e / BM) tiles; tile i of the flat list
// starts at row tile_row[i] of expert tile_expert[i].  Experts with no rows own no tile, so their
// weights are never touched.  One block of 1024 threads, thread e handles expert e, e + 1024, ...
// (E <= 1024 here, so one expert per thread).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void tile_map_kernel(const int32_t *__restrict__ offsets, int E, int BM,
                                                        int32_t *__restrict__ tile_expert,
                                                        int32_t *__restrict__ tile_row,
                                                        int32_t *__restrict__ num_tiles, int max_m_tiles,
                                                        const int32_t *__restrict__ stage_of, int stage)
{
    __shared__ int wave_tot[16];
    const int e = threadIdx.x;
    int row0 = 0, row1 = 0;
    if (e < E && (!stage_of || stage_of[e] == stage)) {
        row0 = offsets[e];
        row1 = offsets[e + 1];
    }
    const int nt = (row1 > row0) ? (row1 - row0 + BM - 1) / BM : 0;
    int incl = nt;
    const int lane = threadIdx.x % kWave;
    const int wave = threadIdx.x / kWave;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int up = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += up;
    }
    if (lane == kWave - 1) wave_tot[wave] = incl;
    __syncthreads();
    int wbase = 0;
    for (int w2 = 0; w2 < wave; ++w2) wbase += wave_tot[w2];
    const int first = wbase + incl - nt;
    for (int i = 0; i < nt; ++i) {
        const int ti = first + i;
        if (ti < max_m_tiles) {  // cannot fail when offsets are consistent with the host's bound
            tile_expert[ti] = e;
            tile_row[ti] = row0 + i * BM;
        }
    }
    if (threadIdx.x == 1023) num_tiles[0] = min(first + nt, max_m_tiles);
}

int launch_tile_map(const int32_t *offsets, int E, int block_m, int32_t *tile_expert, int32_t *tile_row,
                    int32_t *num_tiles, int max_m_tiles, const int32_t *stage_of, int stage, hipStream_t s)
{
    ProfScope ps("tile_map", s);
    hipLaunchKernelGGL(tile_map_kernel, dim3(1), dim3(1024), 0, s, offsets, E, block_m, tile_expert, tile_row,
                       num_tiles, max_m_tiles, stage_of, stage);
    MOE_LAUNCH_CHECK("tile_map_kernel");
    return MOE_OK;
}

}  // namespace moe355
