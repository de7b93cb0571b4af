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

template <bool BF16>
__global__ __launch_bounds__(kThreads) void combine_kernel(const uint4 *__restrict__ yp,
                                                           const int32_t *__restrict__ dst_row,
                                                           const float *__restrict__ w, int64_t total, int vpr,
                                                           int k, uint4 *__restrict__ y)
{
    const int64_t base = (int64_t)blockIdx.x * (kThreads * kUnroll) + threadIdx.x;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t v = base + (int64_t)u * kThreads;
        if (v >= total) continue;
        const int64_t t = v / vpr;
        const int c = (int)(v - t * vpr);
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
        for (int j = 0; j < k; ++j) {
            const int64_t r = dst_row[t * k + j];
            if (r < 0) continue;  // an assignment dropped by a static capacity contributes nothing
            const float g = w[t * k + j];
            const uint4 q = yp[r * vpr + c];
            if (BF16) {
                const uint32_t p[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc[2 * i] = fmaf(g, bf16_lo(p[i]), acc[2 * i]);
                    acc[2 * i + 1] = fmaf(g, bf16_hi(p[i]), acc[2 * i + 1]);
                }
            } else {
                acc[0] = fmaf(g, __uint_as_float(q.x), acc[0]);
                acc[1] = fmaf(g, __uint_as_float(q.y), acc[1]);
                acc[2] = fmaf(g, __uint_as_float(q.z), acc[2]);
                acc[3] = fmaf(g, __uint_as_float(q.w), acc[3]);
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
        y[v] = o;
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
    if (dtype == MOE_DTYPE_BF16)
        hipLaunchKernelGGL((combine_kernel<true>), dim3((unsigned)blocks), dim3(kThreads), 0, s, (const uint4 *)yp,
                           dst_row, w, total, vpr, k, (uint4 *)y);
    else
        hipLaunchKernelGGL((combine_kernel<false>), dim3((unsigned)blocks), dim3(kThreads), 0, s, (const uint4 *)yp,
                           dst_row, w, total, vpr, k, (uint4 *)y);
    MOE_LAUNCH_CHECK("combine_kernel");
    return MOE_OK;
}

}  // namespace moe355
