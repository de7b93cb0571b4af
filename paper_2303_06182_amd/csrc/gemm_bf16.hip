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
// chunk position c ^ ((r >> 1) & 7).  gfx950's LDS serves a 16-byte-per-lane read 16 consecutive
// lanes (256 B, 64 banks) per clock: the 16 rows such a group reads at one K chunk are 8 even rows
// (first half of the banks) and 8 odd rows (second half), and the swizzle gives each half 8
// different chunk positions, so fragment reads are conflict free (measured: 4 clk per
// ds_read_b128 against 6 clk with an (r & 7) swizzle); the 16 chunks two rows' writers store are
// 256 contiguous bytes.
//
// Pipeline: double-buffered LDS; the loads of K-tile kt+1 go straight from global memory into the
// other LDS stage (no register staging) and are issued before the MFMAs of K-tile kt; one barrier
// per K-tile.
//
// Launch: 1-D grid.  Workgroups are handed to the 8 XCDs round-robin, each XCD has its own L2, so
// the block id is first remapped to give every XCD a contiguous range of logical tiles; inside
// the range tiles are ordered GM M-tiles at a time across all N-tiles, so tiles that run together
// on an XCD share A rows and B (weight) rows.
#include <stdlib.h>

#include "moe_internal.h"

namespace moe355 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) void glb_void;

static constexpr int BK = 64;
static constexpr int GROUP_M = 4;

__device__ __forceinline__ uint16_t to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float from_bf16(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

template <int BM, int BN, int WM, int WN, bool OUT_F32, bool RELU, bool GROUPED, bool KFULL>
__global__ __launch_bounds__(WM *WN * 64) void gemm_bf16_kernel(GemmParams p)
{
    constexpr int THREADS = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int MI = WTM / 32, NI = WTN / 32;
    constexpr int A_IT = BM * 8 / THREADS, B_IT = BN * 8 / THREADS;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be made of 32x32 blocks");
    static_assert((BM * 8) % THREADS == 0 && (BN * 8) % THREADS == 0, "tile rows must split evenly over threads");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem_raw[];
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
    const int swz = (lane >> 1) & 7;  // == (row >> 1) & 7 for every row this lane reads
    const int KT = (K + BK - 1) / BK;

    // MFMAs of one K tile out of LDS stage `cur`; the fragments of K-step ks+1 are fetched while
    // the MFMAs of K-step ks run.
    auto compute = [&](int cur) {
        const uint16_t *cA = sA + cur * BM * BK + (wm * WTM + frag_row) * BK;
        const uint16_t *cB = sB + cur * BN * BK + (wn * WTN + frag_row) * BK;
        bf16x8 af[2][MI], bfr[2][NI];
        auto load_frags = [&](int ks, int set) {
            const int chunk = ((ks * 2 + frag_half) ^ swz) << 3;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                af[set][mi] = *reinterpret_cast<const bf16x8 *>(cA + mi * 32 * BK + chunk);
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                bfr[set][ni] = *reinterpret_cast<const bf16x8 *>(cB + ni * 32 * BK + chunk);
        };
        load_frags(0, 0);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            if (ks + 1 < BK / 16) load_frags(ks + 1, (ks + 1) & 1);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][mi], bfr[ks & 1][ni], acc[mi][ni],
                                                                          0, 0, 0);
        }
    };

    if constexpr (KFULL) {
        // ---- global -> LDS without registers (global_load_lds_dwordx4): one instruction moves 64
        // lanes x 16 B = 1 KB = 8 tile rows straight into LDS, lane L landing at byte 16*L of the
        // instruction's LDS base.  The base is fixed per instruction, so the swizzle is applied on
        // the global side: the lane that lands in chunk slot (L & 7) of row r fetches K chunk
        // (L & 7) ^ ((r >> 1) & 7).  Instruction i of wave w fills rows (w*IT + i)*8 .. +7.
        // The loads of K tile kt+1 are issued before the MFMAs of K tile kt and are waited for
        // (vmcnt) only at the barrier that ends the iteration.
        const uint16_t *a_ptr[A_IT];
        const uint16_t *b_ptr[B_IT];
#pragma unroll
        for (int i = 0; i < A_IT; ++i) {
            const int r = (wave * A_IT + i) * 8 + (lane >> 3);
            const int kc = (lane & 7) ^ ((r >> 1) & 7);
            const int gr = min(row0 + r, row_end - 1);  // rows past the end repeat the last one (never stored)
            a_ptr[i] = Ag + (int64_t)gr * p.lda + kc * 8;
        }
#pragma unroll
        for (int i = 0; i < B_IT; ++i) {
            const int r = (wave * B_IT + i) * 8 + (lane >> 3);
            const int kc = (lane & 7) ^ ((r >> 1) & 7);
            const int gn = min(n0 + r, p.N - 1);
            b_ptr[i] = Bg + (int64_t)gn * p.ldb + kc * 8;
        }
        auto issue = [&](int kt, int buf) {
#pragma unroll
            for (int i = 0; i < A_IT; ++i)
                __builtin_amdgcn_global_load_lds((const glb_void *)(a_ptr[i] + kt * BK),
                                                 (lds_void *)(sA + buf * BM * BK + (wave * A_IT + i) * 8 * BK), 16, 0, 0);
#pragma unroll
            for (int i = 0; i < B_IT; ++i)
                __builtin_amdgcn_global_load_lds((const glb_void *)(b_ptr[i] + kt * BK),
                                                 (lds_void *)(sB + buf * BN * BK + (wave * B_IT + i) * 8 * BK), 16, 0, 0);
        };
        issue(0, 0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        for (int kt = 0; kt < KT; ++kt) {
            const int cur = kt & 1;
            if (kt + 1 < KT) issue(kt + 1, cur ^ 1);
            compute(cur);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        }
    } else {
        // ---- K not a multiple of the K tile: stage through registers so the tail can be zero filled.
        // chunk c = tid + i*THREADS; row = c >> 3, kc = c & 7
        const uint16_t *a_ptr[A_IT];
        const uint16_t *b_ptr[B_IT];
        int a_lds[A_IT], b_lds[B_IT];
        const int kc = tid & 7;
#pragma unroll
        for (int i = 0; i < A_IT; ++i) {
            const int r = (tid + i * THREADS) >> 3;
            const int gr = min(row0 + r, row_end - 1);
            a_ptr[i] = Ag + (int64_t)gr * p.lda + kc * 8;
            a_lds[i] = r * BK + ((kc ^ ((r >> 1) & 7)) << 3);
        }
#pragma unroll
        for (int i = 0; i < B_IT; ++i) {
            const int r = (tid + i * THREADS) >> 3;
            const int gn = min(n0 + r, p.N - 1);
            b_ptr[i] = Bg + (int64_t)gn * p.ldb + kc * 8;
            b_lds[i] = r * BK + ((kc ^ ((r >> 1) & 7)) << 3);
        }
        uint4 a_reg[A_IT], b_reg[B_IT];
        auto load_global = [&](int kt) {
            const int k0 = kt * BK;
            const bool ok = k0 + kc * 8 < K;
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
        load_global(0);
        store_lds(0);
        __syncthreads();
        for (int kt = 0; kt < KT; ++kt) {
            const int cur = kt & 1;
            if (kt + 1 < KT) load_global(kt + 1);
            compute(cur);
            if (kt + 1 < KT) store_lds(cur ^ 1);
            __syncthreads();
        }
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

template <int BM, int BN, int WM, int WN, bool OUT_F32, bool RELU, bool GROUPED, bool KFULL>
static int launch_k(const GemmParams &p, hipStream_t s)
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
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN, OUT_F32, RELU, GROUPED, KFULL>;
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

template <int BM, int BN, int WM, int WN, bool OUT_F32, bool RELU, bool GROUPED>
static int launch_one(const GemmParams &p, hipStream_t s)
{
    // K a multiple of the K tile: no per-load tail predicate in the main loop
    return (p.K % BK == 0) ? launch_k<BM, BN, WM, WN, OUT_F32, RELU, GROUPED, true>(p, s)
                           : launch_k<BM, BN, WM, WN, OUT_F32, RELU, GROUPED, false>(p, s);
}

// Tile shapes of the grouped GEMM.  variant -> (BM, BN, waves)
//   1: 128x128, 4 waves   2: 64x128, 4 waves   3: 32x128, 4 waves
//   4: 256x256, 4 waves   5: 256x256, 8 waves  6: 256x128, 4 waves   7: 128x256, 4 waves
static int forced_variant()
{
    static int v = -1;
    if (v < 0) {
        const char *e = getenv("MOE355_GEMM_VARIANT");  // tuning override, 0 / unset = automatic
        v = e ? atoi(e) : 0;
        if (v < 0 || v > 7) v = 0;
    }
    return v;
}

static int variant_block_m(int v)
{
    switch (v) {
    case 1: case 7: return 128;
    case 2: return 64;
    case 3: return 32;
    default: return 256;
    }
}

static int pick_variant(int64_t n_rows, int E)
{
    const int f = forced_variant();
    if (f) return f;
    const int64_t avg = E > 0 ? n_rows / E : n_rows;
    if (avg >= 96) return 1;
    if (avg >= 48) return 2;
    return 3;
}

int gemm_bf16_block_m(int64_t n_rows, int E) { return variant_block_m(pick_variant(n_rows, E)); }

template <int BM, int BN, int WM, int WN>
static int launch_grouped(const GemmParams &p, bool relu, hipStream_t s)
{
    return relu ? launch_one<BM, BN, WM, WN, false, true, true>(p, s)
                : launch_one<BM, BN, WM, WN, false, false, true>(p, s);
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
    int v = forced_variant();
    if (!v || variant_block_m(v) != block_m) v = block_m == 128 ? 1 : block_m == 64 ? 2 : block_m == 32 ? 3 : 4;
    switch (v) {
    case 1: return launch_grouped<128, 128, 2, 2>(p, relu, s);
    case 2: return launch_grouped<64, 128, 1, 4>(p, relu, s);
    case 3: return launch_grouped<32, 128, 1, 4>(p, relu, s);
    case 4: return launch_grouped<256, 256, 2, 2>(p, relu, s);
    case 5: return launch_grouped<256, 256, 2, 4>(p, relu, s);
    case 6: return launch_grouped<256, 128, 2, 2>(p, relu, s);
    case 7: return launch_grouped<128, 256, 2, 2>(p, relu, s);
    default:
        set_error("unsupported GEMM variant %d", v);
        return MOE_ERR_UNSUPPORTED;
    }
}

}  // namespace moe355
