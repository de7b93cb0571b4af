// fp32 GEMM  C = A * B^T (+ bias, ReLU), plain or grouped, for the fp32 storage type.
//
// Same contract as the bf16 MFMA kernel (see gemm_bf16.hip) but computed with fp32 vector FMAs:
// the fp32 workload of this library is the small accuracy configuration (1e-5 tolerance), whose
// arithmetic must stay plain fp32 multiply-add; it is bound by ALU rate, not by memory.
// Tile 64 x 64 x 16, 256 threads, each thread a 4 x 4 block of C; LDS holds both operands
// K-major so that a thread's 4 rows / 4 columns are one 16-byte LDS read per k.
#include "moe_internal.h"

namespace moe355 {

static constexpr int FBM = 64, FBN = 64, FBK = 16, FPAD = 4;

template <bool RELU, bool GROUPED>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmParams p)
{
    __shared__ __attribute__((aligned(16))) float sA[2][FBK][FBM + FPAD];
    __shared__ __attribute__((aligned(16))) float sB[2][FBK][FBN + FPAD];

    const int n_tiles = (p.N + FBN - 1) / FBN;
    const int mt = blockIdx.x / n_tiles;
    const int nt = blockIdx.x - mt * n_tiles;
    int row0, row_end, expert = 0;
    if (GROUPED) {
        if (mt >= p.num_tiles[0]) return;
        expert = p.tile_expert[mt];
        row0 = p.tile_row[mt];
        row_end = p.offsets[expert + 1];
    } else {
        row0 = mt * FBM;
        row_end = p.M;
        if (row0 >= row_end) return;
    }
    const int n0 = nt * FBN;
    const int K = p.K;
    const float *Ag = static_cast<const float *>(p.A);
    const float *Bg = static_cast<const float *>(p.B) + (int64_t)((GROUPED && p.b_slot) ? p.b_slot[expert] : expert) * p.strideB;

    const int tid = threadIdx.x;
    const int lrow = tid >> 2;  // 0..63: tile row this thread copies
    const int kq = tid & 3;     // which float4 along K
    const float *a_ptr = Ag + (int64_t)min(row0 + lrow, row_end - 1) * p.lda + kq * 4;
    const float *b_ptr = Bg + (int64_t)min(n0 + lrow, p.N - 1) * p.ldb + kq * 4;

    const int ty = tid >> 4, tx = tid & 15;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    const int KT = (K + FBK - 1) / FBK;
    float4 ra, rb;
    auto load_global = [&](int kt) {
        const int k0 = kt * FBK + kq * 4;
        const bool ok = k0 < K;
        ra = ok ? *reinterpret_cast<const float4 *>(a_ptr + kt * FBK) : make_float4(0.f, 0.f, 0.f, 0.f);
        rb = ok ? *reinterpret_cast<const float4 *>(b_ptr + kt * FBK) : make_float4(0.f, 0.f, 0.f, 0.f);
    };
    auto store_lds = [&](int buf) {
        sA[buf][kq * 4 + 0][lrow] = ra.x;
        sA[buf][kq * 4 + 1][lrow] = ra.y;
        sA[buf][kq * 4 + 2][lrow] = ra.z;
        sA[buf][kq * 4 + 3][lrow] = ra.w;
        sB[buf][kq * 4 + 0][lrow] = rb.x;
        sB[buf][kq * 4 + 1][lrow] = rb.y;
        sB[buf][kq * 4 + 2][lrow] = rb.z;
        sB[buf][kq * 4 + 3][lrow] = rb.w;
    };

    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < KT) load_global(kt + 1);
#pragma unroll
        for (int kk = 0; kk < FBK; ++kk) {
            const float4 a4 = *reinterpret_cast<const float4 *>(&sA[cur][kk][ty * 4]);
            const float4 b4 = *reinterpret_cast<const float4 *>(&sB[cur][kk][tx * 4]);
            const float av[4] = {a4.x, a4.y, a4.z, a4.w};
            const float bv[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
        if (kt + 1 < KT) store_lds(cur ^ 1);
        __syncthreads();
    }

    const float *bias = static_cast<const float *>(p.bias);
    if (bias) bias += (int64_t)expert * p.strideBias;
    float *C = static_cast<float *>(p.C);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = row0 + ty * 4 + i;
        if (row >= row_end) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = n0 + tx * 4 + j;
            if (col >= p.N) continue;
            float v = acc[i][j];
            if (bias) v += bias[col];
            if (p.bias_f32) v += p.bias_f32[col];
            if (RELU) v = v > 0.f ? v : 0.f;
            C[(int64_t)row * p.ldc + col] = v;
        }
    }
}

int gemm_f32_block_m() { return FBM; }

int launch_gemm_f32(const GemmParams &p, bool grouped, bool relu, hipStream_t s)
{
    const int n_tiles = ceil_div(p.N, FBN);
    const int m_tiles = grouped ? p.max_m_tiles : ceil_div(p.M, FBM);
    if (m_tiles <= 0 || n_tiles <= 0) return MOE_OK;
    const int64_t grid = (int64_t)m_tiles * n_tiles;
    if (grid > 0x7fffffff) {
        set_error("GEMM grid too large");
        return MOE_ERR_UNSUPPORTED;
    }
    if (grouped) {
        if (relu)
            hipLaunchKernelGGL((gemm_f32_kernel<true, true>), dim3((unsigned)grid), dim3(256), 0, s, p);
        else
            hipLaunchKernelGGL((gemm_f32_kernel<false, true>), dim3((unsigned)grid), dim3(256), 0, s, p);
    } else {
        if (relu)
            hipLaunchKernelGGL((gemm_f32_kernel<true, false>), dim3((unsigned)grid), dim3(256), 0, s, p);
        else
            hipLaunchKernelGGL((gemm_f32_kernel<false, false>), dim3((unsigned)grid), dim3(256), 0, s, p);
    }
    MOE_LAUNCH_CHECK("gemm_f32_kernel");
    return MOE_OK;
}

}  // namespace moe355
