// Row movement of dynamic gating: dispatch (reorder the tokens by the sort index into the
// per-expert batches) and combine (restore the original order, weighted by the gate) --
// paper Sec. 5.1: both are indexing operations of O(S*D), replacing the multiplications with
// one-hot masks of static gating.
//
// Both kernels are pure HBM streams.  A row is cut into 16-byte vectors; work item v of the
// flat index space (token, vector) is handled by one lane, four items per lane so that four
// loads are in flight before the first store.  Dispatch walks the TOKENS (every x row is read
// once and written k times), combine walks the tokens too (k rows read, one written), so the
// traffic is exactly T*D + k*T*D elements in each direction and every access is a full,
// contiguous 16-byte lane access inside a contiguous row.
#include "moe_internal.h"

namespace moe355 {

static constexpr int kThreads = 256;
static constexpr int kUnroll = 4;

// vpr = 16-byte vectors per row (D*2/16 for bf16, D*4/16 for fp32)
__global__ __launch_bounds__(kThreads) void dispatch_kernel(const uint4 *__restrict__ x,
                                                            const int32_t *__restrict__ dst_row, int64_t total,
                                                            int vpr, int k, uint4 *__restrict__ xp)
{
    const int64_t base = (int64_t)blockIdx.x * (kThreads * kUnroll) + threadIdx.x;
    uint4 val[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t v = base + (int64_t)u * kThreads;
        if (v < total) val[u] = x[v];
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t v = base + (int64_t)u * kThreads;
        if (v < total) {
            const int64_t t = v / vpr;
            const int c = (int)(v - t * vpr);
            for (int j = 0; j < k; ++j) {
                const int64_t r = dst_row[t * k + j];
                xp[r * vpr + c] = val[u];
            }
        }
    }
}

__device__ __forceinline__ float bf16_lo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t p) { return __uint_as_float(p & 0xffff0000u); }
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    return f32_to_bf16_rne(lo) | (f32_to_bf16_rne(hi) << 16);
}

// KC: compile-time bound of k (the loop over a token's rows is unrolled, so the index loads of all
// the lane's work items go out first, then all row loads, and only then the arithmetic: two memory
// latencies per lane instead of two per row).  The sum runs in slot order j = 0 .. k-1 whatever KC is.
template <bool BF16, int KC>
__global__ __launch_bounds__(kThreads) void combine_kernel(const uint4 *__restrict__ yp,
                                                           const int32_t *__restrict__ dst_row,
                                                           const float *__restrict__ w, int64_t total, int vpr,
                                                           int k, uint4 *__restrict__ y)
{
    const int64_t base = (int64_t)blockIdx.x * (kThreads * kUnroll) + threadIdx.x;
    int64_t row[kUnroll][KC];
    float gate[kUnroll][KC];
    int col[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t v = base + (int64_t)u * kThreads;
        const int64_t t = v < total ? v / vpr : 0;
        col[u] = v < total ? (int)(v - t * vpr) : 0;
#pragma unroll
        for (int j = 0; j < KC; ++j) {
            const bool on = v < total && j < k;
            row[u][j] = on ? (int64_t)dst_row[t * k + j] : -1;  // a dropped assignment (static capacity) is -1 too
            gate[u][j] = on ? w[t * k + j] : 0.f;
        }
    }
    uint4 q[kUnroll][KC];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
#pragma unroll
        for (int j = 0; j < KC; ++j)
            q[u][j] = row[u][j] >= 0 ? yp[row[u][j] * vpr + col[u]] : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t v = base + (int64_t)u * kThreads;
        if (v >= total) continue;
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
#pragma unroll
        for (int j = 0; j < KC; ++j) {
            if (row[u][j] < 0) continue;  // contributes nothing
            const float g = gate[u][j];
            if (BF16) {
                const uint32_t p[4] = {q[u][j].x, q[u][j].y, q[u][j].z, q[u][j].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc[2 * i] = fmaf(g, bf16_lo(p[i]), acc[2 * i]);
                    acc[2 * i + 1] = fmaf(g, bf16_hi(p[i]), acc[2 * i + 1]);
                }
            } else {
                acc[0] = fmaf(g, __uint_as_float(q[u][j].x), acc[0]);
                acc[1] = fmaf(g, __uint_as_float(q[u][j].y), acc[1]);
                acc[2] = fmaf(g, __uint_as_float(q[u][j].z), acc[2]);
                acc[3] = fmaf(g, __uint_as_float(q[u][j].w), acc[3]);
            }
        }
        uint4 o;
        if (BF16) {
            o.x = pack_bf16(acc[0], acc[1]);
            o.y = pack_bf16(acc[2], acc[3]);
            o.z = pack_bf16(acc[4], acc[5]);
            o.w = pack_bf16(acc[6], acc[7]);
        } else {
            o.x = __float_as_uint(acc[0]);
            o.y = __float_as_uint(acc[1]);
            o.z = __float_as_uint(acc[2]);
            o.w = __float_as_uint(acc[3]);
        }
        // y is written once and read by nobody in this layer: a non-temporal store keeps its 2*T*D bytes from
        // sitting dirty in the caches in front of HBM, where the next kernel's reads would wait for their write-back
        // (measured at T = 65536, D = 2048: the gate kernel of the following step 101 -> 81 us, this kernel +4 us)
        typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_nt;
        const u32x4_nt ov = {o.x, o.y, o.z, o.w};
        __builtin_nontemporal_store(ov, reinterpret_cast<u32x4_nt *>(y + v));
    }
}

static int vectors_per_row(int dtype, int D) { return dtype == MOE_DTYPE_BF16 ? D / 8 : D / 4; }

int launch_dispatch(int dtype, const void *x, const int32_t *dst_row, int T, int D, int k, void *xp, hipStream_t s)
{
    if (T == 0) return MOE_OK;
    const int vpr = vectors_per_row(dtype, D);
    const int64_t total = (int64_t)T * vpr;
    const int64_t blocks = (total + kThreads * kUnroll - 1) / (kThreads * kUnroll);
    ProfScope ps("dispatch", s);
    hipLaunchKernelGGL(dispatch_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, s, (const uint4 *)x, dst_row, total,
                       vpr, k, (uint4 *)xp);
    MOE_LAUNCH_CHECK("dispatch_kernel");
    return MOE_OK;
}

int launch_combine(int dtype, const void *yp, const int32_t *dst_row, const float *w, int T, int D, int k, void *y,
                   hipStream_t s)
{
    if (T == 0) return MOE_OK;
    const int vpr = vectors_per_row(dtype, D);
    const int64_t total = (int64_t)T * vpr;
    const int64_t blocks = (total + kThreads * kUnroll - 1) / (kThreads * kUnroll);
    ProfScope ps("combine", s);
#define MOE_COMBINE(BF, KC)                                                                                      \
    hipLaunchKernelGGL((combine_kernel<BF, KC>), dim3((unsigned)blocks), dim3(kThreads), 0, s, (const uint4 *)yp, \
                       dst_row, w, total, vpr, k, (uint4 *)y)
    const bool bf = dtype == MOE_DTYPE_BF16;
    if (k <= 1) { if (bf) MOE_COMBINE(true, 1); else MOE_COMBINE(false, 1); }
    else if (k <= 2) { if (bf) MOE_COMBINE(true, 2); else MOE_COMBINE(false, 2); }
    else if (k <= 4) { if (bf) MOE_COMBINE(true, 4); else MOE_COMBINE(false, 4); }
    else { if (bf) MOE_COMBINE(true, MOE_MAX_K); else MOE_COMBINE(false, MOE_MAX_K); }
#undef MOE_COMBINE
    MOE_LAUNCH_CHECK("combine_kernel");
    return MOE_OK;
}

}  // namespace moe355
