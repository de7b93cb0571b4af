// bf16 MFMA GEMM  C = A * B^T (+ bias, ReLU)  with fp32 accumulation, plain or grouped.
//
// Serves the three dense contractions of the layer: the gate (x * Wg^T, fp32 logits out), and the
// two grouped expert GEMMs (Xp * W1[e]^T with ReLU, H * W2[e]^T), where every expert multiplies
// exactly the rows dynamic gating gave it (paper Sec. 5.1) -- no capacity padding.
//
// Both operands are K-contiguous, so every MFMA operand fragment (8 consecutive bf16 along K for
// one row) is one 16-byte LDS read.  Tile: BM x BN x 64, WM x WN waves of 64 lanes, each wave owns
// a (BM/WM) x (BN/WN) sub-tile made of 32x32 MFMA blocks (v_mfma_f32_32x32x16_bf16).
//
// LDS layout: tile rows of 64 bf16 = 128 B = 8 chunks of 16 B; chunk c of row r is stored at
// chunk position c ^ (r & 7), so the 8 rows a group of 8 lanes reads at the same K chunk fall
// into 8 different bank groups (no conflict for ds_read_b128), and the 8 chunks of one row
// written by 8 consecutive lanes do too.
//
// Pipeline: double-buffered LDS, global loads of K-tile kt+1 are issued before the MFMAs of
// K-tile kt and written to the other buffer after them; one barrier per K-tile.
//
// Launch: 1-D grid.  Workgroups are handed to the 8 XCDs round-robin, each XCD has its own L2, so
// the block id is first remapped to give every XCD a contiguous range of logical tiles; inside
// the range tiles are ordered GM M-tiles at a time across all N-tiles, so tiles that run together
// on an XCD share A rows and B (weight) rows.
#include "moe_internal.h"

namespace moe355 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

static constexpr int BK = 64;
static constexpr int GROUP_M = 4;

__device__ __forceinline__ uint16_t to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float from_bf16(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

template <int BM, int BN, int WM, int WN, bool OUT_F32, bool RELU, bool GROUPED>
__global__ __launch_bounds__(WM *WN * 64) void gemm_bf16_kernel(GemmParams p)
{
    constexpr int THREADS = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int MI = WTM / 32, NI = WTN / 32;
    constexpr int A_IT = BM * 8 / THREADS, B_IT = BN * 8 / THREADS;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be made of 32x32 blocks");
    static_assert((BM * 8) % THREADS == 0 && (BN * 8) % THREADS == 0, "tile rows must split evenly over threads");

    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    uint16_t *sA = reinterpret_cast<uint16_t *>(smem_raw);  // [2][BM*64]
    uint16_t *sB = sA + 2 * BM * BK;                        // [2][BN*64]

    // ---- which tile ----------------------------------------------------------------------------
    const int n_tiles = (p.N + BN - 1) / BN;
    const int G = gridDim.x;  // multiple of 8
    const int bid = blockIdx.x;
    const int lid = (bid & 7) * (G >> 3) + (bid >> 3);
    const int per_group = GROUP_M * n_tiles;
    const int grp = lid / per_group;
    const int within = lid - grp * per_group;
    const int mt = grp * GROUP_M + (within % GROUP_M);
    const int nt = within / GROUP_M;
    int row0, row_end, expert = 0;
    if (GROUPED) {
        if (mt >= p.num_tiles[0]) return;
        expert = p.tile_expert[mt];
        row0 = p.tile_row[mt];
        row_end = p.offsets[expert + 1];
    } else {
        row0 = mt * BM;
        row_end = p.M;
        if (row0 >= row_end) return;
    }
    const int n0 = nt * BN;
    const int K = p.K;

    const uint16_t *Ag = static_cast<const uint16_t *>(p.A);
    const uint16_t *Bg = static_cast<const uint16_t *>(p.B) + (int64_t)expert * p.strideB;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // ---- global -> LDS copy assignment: chunk c = tid + i*THREADS; row = c >> 3, kc = c & 7 -----
    const uint16_t *a_ptr[A_IT];
    const uint16_t *b_ptr[B_IT];
    int a_lds[A_IT], b_lds[B_IT];
    const int kc = tid & 7;
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
        const int r = (tid + i * THREADS) >> 3;
        const int gr = min(row0 + r, row_end - 1);  // rows past the end repeat the last one (never stored)
        a_ptr[i] = Ag + (int64_t)gr * p.lda + kc * 8;
        a_lds[i] = r * BK + ((kc ^ (r & 7)) << 3);
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
        const int r = (tid + i * THREADS) >> 3;
        const int gn = min(n0 + r, p.N - 1);
        b_ptr[i] = Bg + (int64_t)gn * p.ldb + kc * 8;
        b_lds[i] = r * BK + ((kc ^ (r & 7)) << 3);
    }
    const bool k_full = (K % BK) == 0;
    const int KT = (K + BK - 1) / BK;

    uint4 a_reg[A_IT], b_reg[B_IT];
    auto load_global = [&](int kt) {
        const int k0 = kt * BK;
        const bool ok = k_full || (k0 + kc * 8 < K);
#pragma unroll
        for (int i = 0; i < A_IT; ++i)
            a_reg[i] = ok ? *reinterpret_cast<const uint4 *>(a_ptr[i] + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < B_IT; ++i)
            b_reg[i] = ok ? *reinterpret_cast<const uint4 *>(b_ptr[i] + k0) : make_uint4(0, 0, 0, 0);
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_IT; ++i) *reinterpret_cast<uint4 *>(sA + buf * BM * BK + a_lds[i]) = a_reg[i];
#pragma unroll
        for (int i = 0; i < B_IT; ++i) *reinterpret_cast<uint4 *>(sB + buf * BN * BK + b_lds[i]) = b_reg[i];
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    // fragment read offsets: row = (wave tile) + mi*32 + (lane & 31), K chunk = ks*2 + (lane >> 5)
    const int frag_row = lane & 31;
    const int frag_half = lane >> 5;
    const int swz = lane & 7;  // == row & 7 for every row this lane reads

    load_global(0);
    store_lds(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < KT) load_global(kt + 1);
        const uint16_t *cA = sA + cur * BM * BK + (wm * WTM + frag_row) * BK;
        const uint16_t *cB = sB + cur * BN * BK + (wn * WTN + frag_row) * BK;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int chunk = ((ks * 2 + frag_half) ^ swz) << 3;
            bf16x8 af[MI], bfr[NI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                af[mi] = *reinterpret_cast<const bf16x8 *>(cA + mi * 32 * BK + chunk);
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                bfr[ni] = *reinterpret_cast<const bf16x8 *>(cB + ni * 32 * BK + chunk);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
        }
        if (kt + 1 < KT) store_lds(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue: acc register r of a 32x32 block is row 8*(r/4) + 4*(lane/32) + r%4, column lane%32
    const uint16_t *bias = static_cast<const uint16_t *>(p.bias);
    if (bias) bias += (int64_t)expert * p.strideBias;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int col = n0 + wn * WTN + ni * 32 + (lane & 31);
        if (col >= p.N) continue;
        float badd = 0.f;
        if (bias) badd += from_bf16(bias[col]);
        if (p.bias_f32) badd += p.bias_f32[col];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = row0 + wm * WTM + mi * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row < row_end) {
                    float v = acc[mi][ni][r] + badd;
                    if (RELU) v = v > 0.f ? v : 0.f;
                    if (OUT_F32)
                        static_cast<float *>(p.C)[(int64_t)row * p.ldc + col] = v;
                    else
                        static_cast<uint16_t *>(p.C)[(int64_t)row * p.ldc + col] = to_bf16(v);
                }
            }
        }
    }
}

template <int BM, int BN, int WM, int WN, bool OUT_F32, bool RELU, bool GROUPED>
static int launch_one(const GemmParams &p, hipStream_t s)
{
    const int n_tiles = ceil_div(p.N, BN);
    const int m_tiles = GROUPED ? p.max_m_tiles : ceil_div(p.M, BM);
    if (m_tiles <= 0 || n_tiles <= 0) return MOE_OK;
    const int64_t logical = (int64_t)ceil_div(m_tiles, GROUP_M) * GROUP_M * n_tiles;
    const int64_t grid = align_up(logical, 8);
    if (grid > 0x7fffffff) {
        set_error("GEMM grid too large");
        return MOE_ERR_UNSUPPORTED;
    }
    const size_t smem = (size_t)2 * (BM + BN) * BK * sizeof(uint16_t);
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN, OUT_F32, RELU, GROUPED>;
    if (smem > 48 * 1024) {
        static bool attr_set = false;  // per instantiation
        if (!attr_set) {
            MOE_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
            attr_set = true;
        }
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(WM * WN * 64), smem, s, p);
    MOE_LAUNCH_CHECK("gemm_bf16_kernel");
    return MOE_OK;
}

int gemm_bf16_block_m(int64_t n_rows, int E)
{
    const int64_t avg = E > 0 ? n_rows / E : n_rows;
    if (avg >= 512) return 128;
    if (avg >= 96) return 128;
    if (avg >= 48) return 64;
    return 32;
}

// Dispatch over the instantiated shapes.
int launch_gemm_bf16(const GemmParams &p, bool grouped, int block_m, bool out_f32, bool relu, hipStream_t s)
{
    if (!grouped) {
        // gate: fp32 logits, N = E is small
        if (!out_f32 || relu) {
            set_error("plain bf16 GEMM is only instantiated for fp32 output without ReLU");
            return MOE_ERR_UNSUPPORTED;
        }
        if (p.N <= 32) return launch_one<128, 32, 4, 1, true, false, false>(p, s);
        if (p.N <= 64) return launch_one<128, 64, 2, 2, true, false, false>(p, s);
        return launch_one<128, 128, 2, 2, true, false, false>(p, s);
    }
    if (out_f32) {
        set_error("grouped bf16 GEMM is only instantiated for bf16 output");
        return MOE_ERR_UNSUPPORTED;
    }
    switch (block_m) {
    case 128:
        return relu ? launch_one<128, 128, 2, 2, false, true, true>(p, s)
                    : launch_one<128, 128, 2, 2, false, false, true>(p, s);
    case 64:
        return relu ? launch_one<64, 128, 1, 4, false, true, true>(p, s)
                    : launch_one<64, 128, 1, 4, false, false, true>(p, s);
    case 32:
        return relu ? launch_one<32, 128, 1, 4, false, true, true>(p, s)
                    : launch_one<32, 128, 1, 4, false, false, true>(p, s);
    default:
        set_error("unsupported block_m %d", block_m);
        return MOE_ERR_UNSUPPORTED;
    }
}

}  // namespace moe355
