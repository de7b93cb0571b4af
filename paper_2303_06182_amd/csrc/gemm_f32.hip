// fp32 GEMM  C = A * B^T (+ bias, ReLU), plain or grouped, for the fp32 storage type.
//
// Same contract as the bf16 kernel (see gemm_bf16.hip), computed in plain fp32: the fp32 workload of
// this library is the small accuracy configuration (1e-5 tolerance).  Two kernels:
//  * gemm_f32_mfma_kernel (K a multiple of 32, rows 16-byte aligned): 64 x 64 x 32 tile, four waves of
//    32 x 32 outputs each on v_mfma_f32_32x32x2_f32 (fp32 products, fp32 accumulation).  Operand rows
//    are 128 bytes per K tile, laid out in LDS like the bf16 kernel's (16-byte chunk c of row r at chunk
//    position c ^ ((r >> 1) & 7): conflict-free 16-byte fragment reads), filled by global_load_lds_dwordx4
//    three stages deep.  One 16-byte fragment read feeds four MFMAs: the instruction contracts over two
//    k slots per step, lanes 0-31 supplying one and lanes 32-63 the other, and WHICH k a slot stands for
//    is free as long as both operands agree -- so the lower lanes take chunk 2j, the upper lanes chunk
//    2j + 1, and the four floats of a chunk are four steps.
//  * gemm_f32_kernel (any K): 64 x 64 x 16 tile, 4 x 4 outputs per thread, vector FMAs.
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


typedef __attribute__((address_space(3))) void lds_void_f;
typedef __attribute__((address_space(1))) void glb_void_f;
typedef float floatx16 __attribute__((ext_vector_type(16)));
// Fragment reads go through a vector type: an LDS read that carries type-based alias information (float4 is a
// struct of floats) is ordered by the compiler after every direct-to-LDS load in flight (vmcnt(0) in front of
// the read), which would undo the pipeline; the explicit vmcnt before each barrier is what orders them.
typedef float floatx4 __attribute__((ext_vector_type(4)));

static constexpr int MBM = 64, MBN = 64, MBK = 32, MSTAGES = 3;

template <bool RELU, bool GROUPED>
__global__ __launch_bounds__(256) void gemm_f32_mfma_kernel(GemmParams p)
{
    // [stage][A rows 0..63 | B rows 0..63][32 floats], chunk-swizzled
    extern __shared__ __attribute__((aligned(1024))) float smem_dyn[];
    float (*smem)[(MBM + MBN) * MBK] = reinterpret_cast<float (*)[(MBM + MBN) * MBK]>(smem_dyn);

    const int n_tiles = (p.N + MBN - 1) / MBN;
    const int mt = blockIdx.x / n_tiles;
    const int nt = blockIdx.x - mt * n_tiles;
    int row0, row_end, expert = 0;
    if (GROUPED) {
        if (mt >= p.num_tiles[0]) return;
        expert = p.tile_expert[mt];
        row0 = p.tile_row[mt];
        row_end = p.offsets[expert + 1];
    } else {
        row0 = mt * MBM;
        row_end = p.M;
        if (row0 >= row_end) return;
    }
    const int n0 = nt * MBN;
    const float *Ag = static_cast<const float *>(p.A);
    const float *Bg = static_cast<const float *>(p.B) + (int64_t)((GROUPED && p.b_slot) ? p.b_slot[expert] : expert) * p.strideB;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // Loads: one wave instruction fills 8 rows x 128 B of LDS in lane order (lane -> 16 bytes at 16 * lane),
    // so the swizzle is applied on the global side: the lane that fills chunk position cp of row r fetches
    // chunk cp ^ ((r >> 1) & 7).  Wave w fills rows 16 w .. 16 w + 15 of A and of B.  Rows past the end of
    // the batch / of the matrix re-read the last valid row; their products are never stored.
    const float *a_src[2], *b_src[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = wave * 16 + i * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        a_src[i] = Ag + (int64_t)min(row0 + r, row_end - 1) * p.lda + c * 4;
        b_src[i] = Bg + (int64_t)min(n0 + r, p.N - 1) * p.ldb + c * 4;
    }
    auto issue = [&](int kt, int stage) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            __builtin_amdgcn_global_load_lds((const glb_void_f *)(a_src[i] + kt * MBK),
                                             (lds_void_f *)(&smem[stage][(wave * 16 + i * 8) * MBK]), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < 2; ++i)
            __builtin_amdgcn_global_load_lds((const glb_void_f *)(b_src[i] + kt * MBK),
                                             (lds_void_f *)(&smem[stage][(MBM + wave * 16 + i * 8) * MBK]), 16, 0, 0);
    };
    constexpr int LPS = 4;  // load instructions per wave and stage

    // fragment addresses: row lane % 32 of the wave's 32-row block, chunk 2 j + lane / 32
    const int fr = lane & 31, fh = lane >> 5;
    const int ar = wm * 32 + fr, br = MBM + wn * 32 + fr;
    const int a_swz = (ar >> 1) & 7, b_swz = (br >> 1) & 7;

    floatx16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;

    const int KT = p.K / MBK;
    // the loads run MSTAGES - 1 K tiles ahead; past the end they re-read the last K tile into a stage
    // nobody reads any more, so every iteration issues the same number and the vmcnt arithmetic is fixed
#pragma unroll
    for (int i = 0; i < MSTAGES - 1; ++i) issue(min(i, KT - 1), i);
    // s_waitcnt through the builtin (the compiler's wait-count bookkeeping cannot see into inline assembly):
    // vmcnt in bits 3:0, expcnt (bits 6:4) at "no wait", lgkmcnt (bits 11:8) 0 or "no wait"
    constexpr int kWaitStage = ((MSTAGES - 2) * LPS) | (7 << 4);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(kWaitStage | (15 << 8));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    int stage = 0, lstage = MSTAGES - 1;
    for (int kt = 0; kt < KT; ++kt) {
        issue(min(kt + MSTAGES - 1, KT - 1), lstage);  // into the stage the previous iteration read
        lstage = lstage + 1 == MSTAGES ? 0 : lstage + 1;
        const float *sa = &smem[stage][ar * MBK], *sb = &smem[stage][br * MBK];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const floatx4 a4 = *reinterpret_cast<const floatx4 *>(sa + (((2 * j + fh) ^ a_swz) << 2));
            const floatx4 b4 = *reinterpret_cast<const floatx4 *>(sb + (((2 * j + fh) ^ b_swz) << 2));
            // weights first: a lane then owns one output row and 4 x 4 consecutive output columns
#pragma unroll
            for (int q = 0; q < 4; ++q) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(b4[q], a4[q], acc, 0, 0, 0);
        }
        // the K tile read next has landed (this wave's part; the barrier covers the others'), and every
        // fragment read of this stage has returned before another wave may refill it
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(kWaitStage);  // and lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        stage = stage + 1 == MSTAGES ? 0 : stage + 1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no LDS write may outlive the block

    // lane: output row wm*32 + lane%32; register 4 g + i: column wn*32 + 8 g + 4 (lane/32) + i
    const int row = row0 + wm * 32 + fr;
    if (row >= row_end) return;
    const float *bias = static_cast<const float *>(p.bias);
    if (bias) bias += (int64_t)expert * p.strideBias;
    float *c_row = static_cast<float *>(p.C) + (int64_t)row * p.ldc;
    const bool vec_ok = (p.ldc & 3) == 0;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int col = n0 + wn * 32 + g * 8 + fh * 4;
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[i] = acc[g * 4 + i];
            if (col + i < p.N) {
                if (bias) v[i] += bias[col + i];
                if (p.bias_f32) v[i] += p.bias_f32[col + i];
            }
            if (RELU) v[i] = v[i] > 0.f ? v[i] : 0.f;
        }
        if (vec_ok && col + 3 < p.N) {
            *reinterpret_cast<float4 *>(c_row + col) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (col + i < p.N) c_row[col + i] = v[i];
        }
    }
}

// the MFMA kernel's loads are 16 bytes wide and its K loop has no tail
static bool mfma_ok(const GemmParams &p)
{
    return p.K >= MBK && p.K % MBK == 0 && p.lda % 4 == 0 && p.ldb % 4 == 0 && p.strideB % 4 == 0 &&
           reinterpret_cast<uintptr_t>(p.A) % 16 == 0 && reinterpret_cast<uintptr_t>(p.B) % 16 == 0;
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
    const bool mfma = mfma_ok(p);
    constexpr size_t kMfmaLds = (size_t)MSTAGES * (MBM + MBN) * MBK * sizeof(float);
#define MOE355_F32_LAUNCH(R, G)                                                                        \
    do {                                                                                               \
        if (mfma)                                                                                      \
            hipLaunchKernelGGL((gemm_f32_mfma_kernel<R, G>), dim3((unsigned)grid), dim3(256), kMfmaLds, s, p); \
        else                                                                                           \
            hipLaunchKernelGGL((gemm_f32_kernel<R, G>), dim3((unsigned)grid), dim3(256), 0, s, p);      \
    } while (0)
    if (grouped) {
        if (relu)
            MOE355_F32_LAUNCH(true, true);
        else
            MOE355_F32_LAUNCH(false, true);
    } else {
        if (relu)
            MOE355_F32_LAUNCH(true, false);
        else
            MOE355_F32_LAUNCH(false, false);
    }
#undef MOE355_F32_LAUNCH
    MOE_LAUNCH_CHECK("gemm_f32_kernel");
    return MOE_OK;
}

}  // namespace moe355
