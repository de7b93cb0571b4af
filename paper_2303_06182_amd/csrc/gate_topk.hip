// Gate GEMM with the routing decision in its epilogue: logits = x * Wg^T (+ offset) on bf16 MFMAs, and,
// straight from the accumulators, the softmax / top-k of every token and the per-tile expert histogram.
//
// Paper: the gate is a light linear layer (Sec. 2.4) whose only purpose is the top-1 / top-2 decision
// (Sec. 2.3); dynamic gating then counts the occurrences of each expert (Sec. 5.1).  None of the three
// steps needs the [T,E] logits in memory, so with E <= 128 (one column tile) they never leave the
// registers unless the caller asks for them: the kernel streams x once and writes T*k indices and
// weights -- an HBM-bound stream of x.
//
// Tile: BM = 32 * WAVES token rows x BN = 32 * NI experts (all of them) x 64 along D; every wave owns 32
// rows and ALL columns, as NI blocks of v_mfma_f32_32x32x16_bf16 with the gate weights as first operand:
// lane l then holds, for token row (l & 31), the columns 32 ni + 8 g + 4 (l >> 5) + i in accumulator
// 4 g + i of block ni.  A token's E logits therefore sit in exactly two lanes (l and l ^ 32), 16 * NI
// each, in ascending column order: the k rounds of "largest remaining logit, ties to the lower expert"
// run inside the lane and finish with one exchange between the two.
//
// K pipeline: STAGES LDS stages filled by global_load_lds_dwordx4 (no register staging), STAGES - 1 K
// tiles in flight; rows of 128 B, 16-byte chunk c of row r at chunk slot c ^ ((r >> 1) & 7) (conflict-free
// fragment reads on gfx950's 64-bank LDS), the swizzle applied on the global side of the load.  A block
// is one tile (no persistence: the epilogue is short and there is nothing to keep resident); the tile
// height is chosen so that the launch still has a tile per CU.
// (Measured at T = 65536, D = 2048, E = 128 on MI355X: 50 us when x is partly served by the last-level cache,
// 78 us when every launch reads a different copy of x, about 100 us inside the layer behind the previous
// step's writes.  A bare read of x in the same order -- a CU owning 256 consecutive rows, no arithmetic --
// takes 57 us cold, whatever the bytes per row visit (128 B .. 1 KB) or the depth of the prefetch.  A variant
// that keeps the x rows out of LDS -- each lane loading its own fragments straight into registers four K
// tiles ahead, only the gate weights staged -- measured the same cold and 20 % slower warm, and was dropped.)
#include <mutex>

#include "moe_internal.h"

namespace moe355 {

typedef __attribute__((ext_vector_type(8))) __bf16 gt_bf16x8;
typedef __attribute__((ext_vector_type(16))) float gt_f32x16;
typedef __attribute__((address_space(3))) void gt_lds_void;
typedef __attribute__((address_space(1))) void gt_glb_void;

struct GateTopkParams {
    const uint16_t *x;    // [T, K] bf16
    const uint16_t *wg;   // [E, K] bf16
    const float *bias;    // [E] fp32 or NULL
    float *logits;        // [T, E] fp32 or NULL
    int32_t *idx;         // [T, k]
    float *w;             // [T, k]
    int32_t *hist;        // [tiles, E] or NULL: hist[tile, e] = assignments of the tile's tokens to expert e
    int T, E, K, k, renorm;
};

template <int WAVES, int NI, int STAGES>
__global__ __launch_bounds__(WAVES * 64) void gate_topk_kernel(GateTopkParams p)
{
    constexpr int THREADS = WAVES * 64;
    constexpr int BM = 32 * WAVES, BN = 32 * NI, BK = 64;
    constexpr int A_IT = 4;                // 1 KB load instructions per wave and stage: BM / 8 rows-of-8 over WAVES waves
    constexpr int B_IT = NI * 4 / WAVES;   // BN / 8 over WAVES waves
    static_assert((NI * 4) % WAVES == 0, "the gate weight tile must split evenly over the waves");
    static_assert(STAGES >= 2 && STAGES <= 4, "two to four LDS stages");
    constexpr int LPS = A_IT + B_IT;
    constexpr int NS = NI * 16;            // logits a lane holds
    static_assert(NS <= 64, "the taken-mask is 64 bits");

    extern __shared__ __attribute__((aligned(1024))) uint8_t gt_smem[];
    uint16_t *sA = reinterpret_cast<uint16_t *>(gt_smem);  // [STAGES][BM * 64]
    uint16_t *sB = sA + STAGES * BM * BK;                   // [STAGES][BN * 64]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int row0 = blockIdx.x * BM;
    const int K = p.K, T = p.T, E = p.E;
    const int KT = K / BK;  // the launcher checked that K is a multiple of the K tile

    // ---- global -> LDS: instruction i of wave w fills tile rows (w * IT + i) * 8 .. + 7; lane L lands in row
    // (L >> 3), chunk slot (L & 7) and fetches K chunk (L & 7) ^ ((row >> 1) & 7).  Rows past the end of x or
    // Wg repeat the last one (their results are never used).
    const uint16_t *a_ptr[A_IT];
    const uint16_t *b_ptr[B_IT];
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
        const int r = (wave * A_IT + i) * 8 + (lane >> 3);
        const int kc = (lane & 7) ^ ((r >> 1) & 7);
        const int gr = min(row0 + r, T - 1);
        a_ptr[i] = p.x + (int64_t)gr * K + kc * 8;
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
        const int r = (wave * B_IT + i) * 8 + (lane >> 3);
        const int kc = (lane & 7) ^ ((r >> 1) & 7);
        const int gn = min(r, E - 1);
        b_ptr[i] = p.wg + (int64_t)gn * K + kc * 8;
    }
    auto issue = [&](int kt, int buf) {
#pragma unroll
        for (int i = 0; i < A_IT; ++i)
            __builtin_amdgcn_global_load_lds((const gt_glb_void *)(a_ptr[i] + kt * BK),
                                             (gt_lds_void *)(sA + buf * BM * BK + (wave * A_IT + i) * 8 * BK), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < B_IT; ++i)
            __builtin_amdgcn_global_load_lds((const gt_glb_void *)(b_ptr[i] + kt * BK),
                                             (gt_lds_void *)(sB + buf * BN * BK + (wave * B_IT + i) * 8 * BK), 16, 0, 0);
    };
    // "at most STAGES - 2 stages' loads of this wave outstanding": the K tile needed next has landed.  Every
    // iteration issues the same number of loads (past the end it re-reads the last K tile into a stage nobody
    // reads any more), which keeps this arithmetic fixed.
    constexpr int WAITN = (STAGES - 2) * LPS;
    static_assert(WAITN < 64, "vmcnt is a 6-bit counter");
    auto wait_loads = [&]() {
        constexpr int kWaitImm = (WAITN & 15) | ((WAITN >> 4) << 14) | (7 << 4) | (15 << 8);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(kWaitImm);
        asm volatile("" ::: "memory");
    };
    auto block_barrier = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    };

    gt_f32x16 acc[NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[ni][r] = 0.f;

    const int frag_row = lane & 31;
    const int half = lane >> 5;
    const int swz = (lane >> 1) & 7;  // == (row >> 1) & 7 for every tile row this lane reads

#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) issue(min(s, KT - 1), s);
    int cur = 0, nxt = STAGES - 1;
    for (int kt = 0; kt < KT; ++kt) {
        wait_loads();
        block_barrier();  // stage `cur` is complete for every wave; everybody is done reading stage `nxt`
        issue(min(kt + STAGES - 1, KT - 1), nxt);
        const uint16_t *cA = sA + cur * BM * BK + (wave * 32 + frag_row) * BK;
        const uint16_t *cB = sB + cur * BN * BK + frag_row * BK;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int chunkpos = ((ks * 2 + half) ^ swz) << 3;
            const gt_bf16x8 af = *reinterpret_cast<const gt_bf16x8 *>(cA + chunkpos);
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const gt_bf16x8 bf = *reinterpret_cast<const gt_bf16x8 *>(cB + ni * 32 * BK + chunkpos);
                acc[ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf, af, acc[ni], 0, 0, 0);
            }
        }
        cur = (cur + 1 == STAGES) ? 0 : cur + 1;
        nxt = (nxt + 1 == STAGES) ? 0 : nxt + 1;
    }
    // no load may still be writing LDS when the histogram reuses it
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    block_barrier();

    // ---- epilogue: this lane's logits in ascending column order
    const int row = row0 + wave * 32 + frag_row;
    const bool live = row < T;
    auto col_of = [&](int s) { return (s >> 4) * 32 + ((s >> 2) & 3) * 8 + 4 * half + (s & 3); };
    float v[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) v[s] = acc[s >> 4][s & 15];
    if (p.bias) {  // uniform over the grid.  All offsets are requested before the first is added (columns past E read
                   // the last one): a load per column behind its own predicate makes 16 * NI dependent memory latencies
        float off[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s) off[s] = p.bias[min(col_of(s), E - 1)];
#pragma unroll
        for (int s = 0; s < NS; ++s) v[s] += off[s];
    }
    if (p.logits && live) {
        float *dst = p.logits + (int64_t)row * E;
        if ((E & 3) == 0) {
#pragma unroll
            for (int q = 0; q < NS / 4; ++q) {
                const int c = col_of(4 * q);
                if (c < E) *reinterpret_cast<float4 *>(dst + c) = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
            }
        } else {
#pragma unroll
            for (int s = 0; s < NS; ++s)
                if (col_of(s) < E) dst[col_of(s)] = v[s];
        }
    }

    const float NEG_INF = -__builtin_huge_valf();
    constexpr int NONE = 0x7fffffff;
    uint64_t taken = 0;  // bit s: slot s already selected, or past the last expert
#pragma unroll
    for (int s = 0; s < NS; ++s)
        if (col_of(s) >= E) taken |= 1ull << s;

    float sel_v[MOE_MAX_K];
    int sel_e[MOE_MAX_K];
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j) {
        sel_v[j] = NEG_INF;
        sel_e[j] = 0;
        if (j >= p.k) continue;  // uniform over the grid
        float bv = NEG_INF;
        int bs = -1;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const bool free_slot = !((taken >> s) & 1ull);
            if (free_slot && (bs < 0 || v[s] > bv)) {  // strict: the first (lowest) column keeps a tie
                bv = v[s];
                bs = s;
            }
        }
        int be = bs >= 0 ? col_of(bs) : NONE;
        // the other half of the row: (value desc, column asc) decides
        const float ov = __shfl_xor(bv, 32, 64);
        const int oe = __shfl_xor(be, 32, 64);
        if (oe != NONE && (be == NONE || ov > bv || (ov == bv && oe < be))) {
            bv = ov;
            be = oe;
        }
        // both lanes agree for finite inputs; take the lower lane's view so that the bookkeeping stays
        // consistent whatever the inputs are
        bv = __shfl(bv, frag_row, 64);
        be = __shfl(be, frag_row, 64);
        sel_v[j] = bv;
        sel_e[j] = be == NONE ? 0 : be;
        if (be != NONE && ((be >> 2) & 1) == half) {  // the column lives in this lane: mark its slot
            const int s_own = (be >> 5) * 16 + ((be >> 3) & 3) * 4 + (be & 3);
            taken |= 1ull << s_own;
        }
    }

    // gate weights in fp32: exp(l - max) over the selected (renormalised) or over all experts
    const float m = sel_v[0];
    float denom = 0.f;
    if (p.renorm) {
#pragma unroll
        for (int j = 0; j < MOE_MAX_K; ++j)
            if (j < p.k) denom += expf(sel_v[j] - m);
    } else {
        float part = 0.f;
#pragma unroll
        for (int s = 0; s < NS; ++s)
            if (col_of(s) < E) part += expf(v[s] - m);
        denom = part + __shfl_xor(part, 32, 64);
    }
    if (live && half == 0) {
#pragma unroll
        for (int j = 0; j < MOE_MAX_K; ++j) {
            if (j < p.k) {
                p.idx[(int64_t)row * p.k + j] = sel_e[j];
                p.w[(int64_t)row * p.k + j] = expf(sel_v[j] - m) / denom;
            }
        }
    }

    // ---- the tile's expert histogram (LDS atomics on integers: the sums do not depend on the order)
    if (p.hist) {
        int *hist = reinterpret_cast<int *>(gt_smem);
        for (int e = tid; e < E; e += THREADS) hist[e] = 0;
        __syncthreads();
        if (live && half == 0) {
#pragma unroll
            for (int j = 0; j < MOE_MAX_K; ++j)
                if (j < p.k) atomicAdd(&hist[sel_e[j]], 1);
        }
        __syncthreads();
        for (int e = tid; e < E; e += THREADS) p.hist[(int64_t)blockIdx.x * E + e] = hist[e];
    }
}

template <int WAVES, int NI, int STAGES>
static int launch_gate_topk_t(const GateTopkParams &p, hipStream_t s)
{
    constexpr int BM = 32 * WAVES, BN = 32 * NI;
    const size_t smem = (size_t)STAGES * (BM + BN) * 64 * sizeof(uint16_t);
    auto kern = gate_topk_kernel<WAVES, NI, STAGES>;
    static std::once_flag once;  // per instantiation
    static hipError_t attr_rc = hipSuccess;
    std::call_once(once, [&]() {
        attr_rc = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)smem);
    });
    MOE_HIP_CHECK(attr_rc);
    ProfScope ps("gate_topk", s);
    hipLaunchKernelGGL(kern, dim3((unsigned)ceil_div(p.T, BM)), dim3(WAVES * 64), smem, s, p);
    MOE_LAUNCH_CHECK("gate_topk_kernel");
    return MOE_OK;
}

bool gate_topk_fused_ok(int dtype, int T, int E, int K)
{
    return dtype == MOE_DTYPE_BF16 && T > 0 && E >= 1 && E <= 128 && K >= 64 && K % 64 == 0;
}

// Tokens per tile (= tokens per histogram row) the fused kernel uses for T tokens and E experts: the tallest
// of 256, 128, 64, 32 rows that still gives every CU a tile and whose wave count divides the weight tile's
// load instructions.
int gate_topk_tile_tokens(int T, int E, int num_cus)
{
    const int ni = ceil_div(E, 32);
    for (int waves = 8; waves > 1; waves >>= 1) {
        if ((ni * 4) % waves != 0) continue;
        if (ceil_div(T, 32 * waves) >= num_cus) return 32 * waves;
    }
    return 32;
}

int launch_gate_topk(const void *x, const void *wg, const float *gate_bias, int T, int E, int K, int k, int renorm,
                     float *logits, int32_t *idx, float *w, int32_t *hist, int num_cus, hipStream_t s)
{
    GateTopkParams p;
    p.x = static_cast<const uint16_t *>(x);
    p.wg = static_cast<const uint16_t *>(wg);
    p.bias = gate_bias;
    p.logits = logits;
    p.idx = idx;
    p.w = w;
    p.hist = hist;
    p.T = T;
    p.E = E;
    p.K = K;
    p.k = k;
    p.renorm = renorm;
    const int ni = ceil_div(E, 32);
    const int waves = gate_topk_tile_tokens(T, E, num_cus) / 32;
#define MOE_GT(W, N, S) return launch_gate_topk_t<W, N, S>(p, s)
    switch (waves * 10 + ni) {
    case 84: MOE_GT(8, 4, 3);
    case 82: MOE_GT(8, 2, 3);
    case 44: MOE_GT(4, 4, 3);
    case 43: MOE_GT(4, 3, 3);
    case 42: MOE_GT(4, 2, 3);
    case 41: MOE_GT(4, 1, 3);
    case 24: MOE_GT(2, 4, 3);
    case 23: MOE_GT(2, 3, 3);
    case 22: MOE_GT(2, 2, 3);
    case 21: MOE_GT(2, 1, 3);
    case 14: MOE_GT(1, 4, 4);
    case 13: MOE_GT(1, 3, 4);
    case 12: MOE_GT(1, 2, 4);
    case 11: MOE_GT(1, 1, 4);
    default: break;
    }
#undef MOE_GT
    set_error("gate_topk: no kernel for %d waves and %d column blocks", waves, ni);
    return MOE_ERR_UNSUPPORTED;
}

}  // namespace moe355
