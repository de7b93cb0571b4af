// Kernels of the static-capacity baseline (paper Sec. 3.2 and Sec. 5.1): every expert owns
// `capacity` rows; an assignment takes the first empty row of its expert in the order "all first
// choices by token, then all second choices, ..." and is dropped when the expert is full; unused
// rows are zero; rows are moved either by index or -- the formulation the paper identifies as the
// inefficiency -- by multiplying with one-hot dispatch masks and weighted combine masks.
//
// The slot of an assignment is its rank inside its expert in slot-major order, which is exactly
// what the dynamic-gating routing kernels compute when they are run on the transposed index array
// with k = 1; the kernels here turn that rank into padded row numbers, masks and zero-padded
// buffers.  The GEMMs are the library's ordinary plain / grouped GEMMs.
#include "moe_internal.h"

namespace moe355 {

static constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void transpose_idx_kernel(const int32_t *__restrict__ idx, int T, int k,
                                                                 int32_t *__restrict__ idx_t,
                                                                 int32_t *__restrict__ dropped)
{
    const int64_t a = (int64_t)blockIdx.x * kThreads + threadIdx.x;  // a = t*k + j
    if (a == 0) dropped[0] = 0;
    if (a >= (int64_t)T * k) return;
    const int64_t t = a / k;
    const int j = (int)(a - t * k);
    idx_t[(int64_t)j * T + t] = idx[a];
}

__global__ __launch_bounds__(kThreads) void static_rows_kernel(const int32_t *__restrict__ idx_t,
                                                               const int32_t *__restrict__ pos,
                                                               const int32_t *__restrict__ offsets_s, int T, int k,
                                                               int E, int capacity, int32_t *__restrict__ slot_row,
                                                               int32_t *__restrict__ dropped)
{
    const int64_t a = (int64_t)blockIdx.x * kThreads + threadIdx.x;  // slot-major: a = j*T + t
    bool drop = false;
    if (a < (int64_t)T * k) {
        const int j = (int)(a / T);
        const int64_t t = a - (int64_t)j * T;
        int e = idx_t[a];
        e = e < 0 ? 0 : (e >= E ? E - 1 : e);
        const int slot = pos[a] - offsets_s[e];
        drop = slot >= capacity;
        slot_row[t * k + j] = drop ? -1 : e * capacity + slot;
    }
    const uint64_t m = __ballot(drop);
    if ((threadIdx.x & 63) == 0 && m) atomicAdd(dropped, __popcll(m));
}

__global__ __launch_bounds__(kThreads) void fill_u32_kernel(uint32_t *__restrict__ dst, int64_t n, uint32_t value)
{
    // 16-byte stores over the aligned body, scalar tail
    const int64_t nvec = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    uint4 v = make_uint4(value, value, value, value);
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += stride)
        reinterpret_cast<uint4 *>(dst)[i] = v;
    for (int64_t i = (nvec << 2) + (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) dst[i] = value;
}

__global__ __launch_bounds__(kThreads) void row_tokens_kernel(const int32_t *__restrict__ slot_row, int64_t n, int k,
                                                              int32_t *__restrict__ row_tok)
{
    const int64_t a = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (a >= n) return;
    const int r = slot_row[a];
    if (r >= 0) row_tok[r] = (int32_t)(a / k);
}

__global__ __launch_bounds__(kThreads) void padded_gather_kernel(const uint4 *__restrict__ x,
                                                                 const int32_t *__restrict__ row_tok, int64_t total,
                                                                 int vpr, uint4 *__restrict__ xd)
{
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (v >= total) return;
    const int64_t r = v / vpr;
    const int c = (int)(v - r * vpr);
    const int t = row_tok[r];
    xd[v] = t >= 0 ? x[(int64_t)t * vpr + c] : make_uint4(0, 0, 0, 0);
}

__global__ void static_offsets_kernel(int32_t *__restrict__ offsets_static, int E, int capacity)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e <= E) offsets_static[e] = e * capacity;
}

template <typename T>
__global__ __launch_bounds__(256) void transpose_pad_kernel(const T *__restrict__ in, int64_t R, int64_t C,
                                                            T *__restrict__ out, int64_t ldo)
{
    __shared__ T tile[32][33];
    const int64_t r0 = (int64_t)blockIdx.y * 32, c0 = (int64_t)blockIdx.x * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    for (int i = ty; i < 32; i += 8) {
        const int64_t r = r0 + i, c = c0 + tx;
        tile[i][tx] = (r < R && c < C) ? in[r * C + c] : T(0);
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
        const int64_t c = c0 + i, r = r0 + tx;  // out[c, r]
        if (c < C && r < ldo) out[c * ldo + r] = tile[tx][i];
    }
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void static_masks_kernel(const int32_t *__restrict__ slot_row,
                                                                const float *__restrict__ w, int64_t n, int k,
                                                                void *__restrict__ mask, int64_t ldm,
                                                                void *__restrict__ cw, int64_t ldc)
{
    const int64_t a = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (a >= n) return;
    const int r = slot_row[a];
    if (r < 0) return;
    const int64_t t = a / k;
    if (BF16) {
        uint32_t u = __float_as_uint(w[a]);
        u += 0x7fffu + ((u >> 16) & 1u);
        static_cast<uint16_t *>(mask)[(int64_t)r * ldm + t] = 0x3f80;  // 1.0
        static_cast<uint16_t *>(cw)[t * ldc + r] = (uint16_t)(u >> 16);
    } else {
        static_cast<float *>(mask)[(int64_t)r * ldm + t] = 1.0f;
        static_cast<float *>(cw)[t * ldc + r] = w[a];
    }
}

static unsigned blocks_for(int64_t n) { return (unsigned)((n + kThreads - 1) / kThreads); }

int launch_transpose_idx(const int32_t *idx, int T, int k, int32_t *idx_t, int32_t *dropped, hipStream_t s)
{
    ProfScope ps("static_slots", s);
    hipLaunchKernelGGL(transpose_idx_kernel, dim3(blocks_for((int64_t)T * k > 0 ? (int64_t)T * k : 1)), dim3(kThreads), 0,
                       s, idx, T, k, idx_t, dropped);
    MOE_LAUNCH_CHECK("transpose_idx_kernel");
    return MOE_OK;
}

int launch_static_rows(const int32_t *idx_t, const int32_t *pos, const int32_t *offsets_s, int T, int k, int E,
                       int capacity, int32_t *slot_row, int32_t *dropped, hipStream_t s)
{
    ProfScope ps("static_slots", s);
    hipLaunchKernelGGL(static_rows_kernel, dim3(blocks_for((int64_t)T * k)), dim3(kThreads), 0, s, idx_t, pos,
                       offsets_s, T, k, E, capacity, slot_row, dropped);
    MOE_LAUNCH_CHECK("static_rows_kernel");
    return MOE_OK;
}

int launch_fill_u32(void *dst, int64_t n_words, uint32_t value, hipStream_t s)
{
    if (n_words <= 0) return MOE_OK;
    ProfScope ps("static_fill", s);
    int64_t blocks = (n_words / 4 + kThreads - 1) / kThreads;
    if (blocks < 1) blocks = 1;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, s, static_cast<uint32_t *>(dst),
                       n_words, value);
    MOE_LAUNCH_CHECK("fill_u32_kernel");
    return MOE_OK;
}

int launch_row_tokens(const int32_t *slot_row, int T, int k, int32_t *row_tok, hipStream_t s)
{
    ProfScope ps("static_slots", s);
    hipLaunchKernelGGL(row_tokens_kernel, dim3(blocks_for((int64_t)T * k)), dim3(kThreads), 0, s, slot_row,
                       (int64_t)T * k, k, row_tok);
    MOE_LAUNCH_CHECK("row_tokens_kernel");
    return MOE_OK;
}

int launch_padded_gather(int dtype, const void *x, const int32_t *row_tok, int64_t rows, int D, void *xd, hipStream_t s)
{
    const int vpr = dtype == MOE_DTYPE_BF16 ? D / 8 : D / 4;
    const int64_t total = rows * vpr;
    if (total == 0) return MOE_OK;
    ProfScope ps("static_dispatch_indexed", s);
    hipLaunchKernelGGL(padded_gather_kernel, dim3(blocks_for(total)), dim3(kThreads), 0, s, (const uint4 *)x, row_tok,
                       total, vpr, (uint4 *)xd);
    MOE_LAUNCH_CHECK("padded_gather_kernel");
    return MOE_OK;
}

int launch_static_offsets(int32_t *offsets_static, int E, int capacity, hipStream_t s)
{
    hipLaunchKernelGGL(static_offsets_kernel, dim3((E + 1 + 255) / 256), dim3(256), 0, s, offsets_static, E, capacity);
    MOE_LAUNCH_CHECK("static_offsets_kernel");
    return MOE_OK;
}

int launch_transpose_pad(int dtype, const void *in, int64_t R, int64_t C, void *out, int64_t ldo, hipStream_t s)
{
    const int64_t rmax = R > ldo ? R : ldo;
    dim3 grid((unsigned)((C + 31) / 32), (unsigned)((rmax + 31) / 32));
    ProfScope ps("static_transpose", s);
    if (dtype == MOE_DTYPE_BF16)
        hipLaunchKernelGGL((transpose_pad_kernel<uint16_t>), grid, dim3(256), 0, s, (const uint16_t *)in, R, C,
                           (uint16_t *)out, ldo);
    else
        hipLaunchKernelGGL((transpose_pad_kernel<uint32_t>), grid, dim3(256), 0, s, (const uint32_t *)in, R, C,
                           (uint32_t *)out, ldo);
    MOE_LAUNCH_CHECK("transpose_pad_kernel");
    return MOE_OK;
}

int launch_static_masks(int dtype, const int32_t *slot_row, const float *w, int T, int k, void *mask, int64_t ldm,
                        void *cw, int64_t ldc, hipStream_t s)
{
    const int64_t n = (int64_t)T * k;
    ProfScope ps("static_masks", s);
    if (dtype == MOE_DTYPE_BF16)
        hipLaunchKernelGGL((static_masks_kernel<true>), dim3(blocks_for(n)), dim3(kThreads), 0, s, slot_row, w, n, k,
                           mask, ldm, cw, ldc);
    else
        hipLaunchKernelGGL((static_masks_kernel<false>), dim3(blocks_for(n)), dim3(kThreads), 0, s, slot_row, w, n, k,
                           mask, ldm, cw, ldc);
    MOE_LAUNCH_CHECK("static_masks_kernel");
    return MOE_OK;
}

}  // namespace moe355
