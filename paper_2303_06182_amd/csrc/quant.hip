// Weight-only 8-bit expert weights (an MI355X-side extension, not part of the paper): W[e] is stored
// as OCP e4m3 bytes with one power-of-two fp32 scale per expert, W[e] ~ scale[e] * q[e].  The scale
// is the smallest power of two s with max|W[e]| / s <= 448 (the largest e4m3 value), so the division
// is exact and nothing saturates; the rounding to e4m3 is the hardware's round-to-nearest-even.
//
// Byte layout of q: not row-major.  The grouped GEMM moves 16 weight rows x 64 K-bytes with one
// load instruction, so exactly that 1 KB block is contiguous, and the blocks of one 16-row group
// follow each other along K:  byte of element (n, k) of a [rows, cols] matrix =
//     ((n / 16) * (cols / 64) + k / 64) * 1024 + (n % 16) * 64 + k % 64.
// A GEMM block then reads a few strictly sequential streams instead of 64-byte slices of rows
// that lie `cols` bytes apart.
#include "moe_internal.h"

namespace moe355 {

static constexpr int kQThreads = 256;

// Four consecutive elements as floats: one 8-byte (bf16) or 16-byte (fp32) load.  i is a multiple of 4.
template <bool BF16>
__device__ __forceinline__ void load4(const void *w, int64_t i, float (&v)[4])
{
    if (BF16) {
        const uint2 r = *reinterpret_cast<const uint2 *>(static_cast<const uint16_t *>(w) + i);
        v[0] = __uint_as_float(r.x << 16);
        v[1] = __uint_as_float(r.x & 0xffff0000u);
        v[2] = __uint_as_float(r.y << 16);
        v[3] = __uint_as_float(r.y & 0xffff0000u);
    } else {
        const float4 r = *reinterpret_cast<const float4 *>(static_cast<const float *>(w) + i);
        v[0] = r.x;
        v[1] = r.y;
        v[2] = r.z;
        v[3] = r.w;
    }
}

// scale[e] <- bit pattern of max |w| over the expert (non-negative floats order like their bits)
template <bool BF16>
__global__ __launch_bounds__(kQThreads) void absmax_kernel(const void *__restrict__ w, int64_t per_expert,
                                                           uint32_t *__restrict__ absmax_bits)
{
    const int e = blockIdx.y;
    float m = 0.f;
    for (int64_t i = ((int64_t)blockIdx.x * kQThreads + threadIdx.x) * 4; i < per_expert;
         i += (int64_t)gridDim.x * kQThreads * 4) {
        float v[4];
        load4<BF16>(w, (int64_t)e * per_expert + i, v);
        m = fmaxf(fmaxf(m, fmaxf(fabsf(v[0]), fabsf(v[1]))), fmaxf(fabsf(v[2]), fabsf(v[3])));
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if ((threadIdx.x & 63) == 0) atomicMax(&absmax_bits[e], __float_as_uint(m));
}

// Smallest power of two s with absmax <= 448 s, without a division: absmax = mant * 2^ex with mant in
// [0.5, 1) and 448 = 0.875 * 2^9.  Kept a normal number so that 1 / s is exact too.
__device__ __forceinline__ float scale_of(float absmax)
{
    if (!(absmax > 0.f)) return 1.f;
    int ex;
    const float mant = frexpf(absmax, &ex);
    int n = (mant <= 0.875f ? ex - 9 : ex - 8);
    n = n < -126 ? -126 : n;
    return ldexpf(1.f, n);
}

template <bool BF16>
__global__ __launch_bounds__(kQThreads) void quantize_kernel(const void *__restrict__ w, int64_t per_expert, int cols,
                                                             const uint32_t *__restrict__ absmax_bits,
                                                             uint8_t *__restrict__ q)
{
    const int e = blockIdx.y;
    const float inv = 1.f / scale_of(__uint_as_float(absmax_bits[e]));  // a power of two: exact
    const int kblocks = cols >> 6;
    // four elements of one row (one 32-bit word of output) per thread and step; cols is a multiple of 64
    for (int64_t i = ((int64_t)blockIdx.x * kQThreads + threadIdx.x) * 4; i < per_expert;
         i += (int64_t)gridDim.x * kQThreads * 4) {
        const int64_t g = (int64_t)e * per_expert + i;
        float v[4];
        load4<BF16>(w, g, v);
        int word = __builtin_amdgcn_cvt_pk_fp8_f32(v[0] * inv, v[1] * inv, 0, false);
        word = __builtin_amdgcn_cvt_pk_fp8_f32(v[2] * inv, v[3] * inv, word, true);
        const int64_t n = i / cols;
        const int k = (int)(i - n * cols);
        const int64_t tiled = ((n >> 4) * kblocks + (k >> 6)) * 1024 + (n & 15) * 64 + (k & 63);
        *reinterpret_cast<int *>(q + (int64_t)e * per_expert + tiled) = word;
    }
}

__global__ void finish_scale_kernel(uint32_t *__restrict__ bits_then_scale, int E)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < E) bits_then_scale[e] = __float_as_uint(scale_of(__uint_as_float(bits_then_scale[e])));
}

// ---- 4-bit weights with block scales (the OCP microscaling layout: e2m1 elements, one e8m0 scale per
// 32 elements along the row) ------------------------------------------------------------------------
// Element values: code & 7 -> 0, 0.5, 1, 1.5, 2, 3, 4, 6; bit 3 is the sign.  The block scale is the
// smallest power of two s with max|block| <= 6 s (so nothing saturates), stored as the byte s = 2^(b - 127),
// b >= 1; an all-zero block gets b = 127.  Rounding to nearest, ties to the even code.
// Byte layouts, both made for the grouped GEMM: data, 32 rows x 64 columns per contiguous 1 KB (row r of
// the block at byte 32 r, two elements per byte, the lower column in the low nibble), the blocks of a
// 32-row group one after the other along the columns; scales, 32 rows x 16 bytes per contiguous 512 B (the
// 16 scales of 512 columns), again group by group along the columns, the last 512-column group padded.
__device__ __forceinline__ uint32_t e2m1_code(float v)
{
    const float a = fabsf(v);
    uint32_t c;
    if (a <= 0.25f) c = 0;
    else if (a < 0.75f) c = 1;
    else if (a <= 1.25f) c = 2;
    else if (a < 1.75f) c = 3;
    else if (a <= 2.5f) c = 4;
    else if (a < 3.5f) c = 5;
    else if (a <= 5.0f) c = 6;
    else c = 7;
    return c | (__float_as_uint(v) >> 31 << 3);
}

template <bool BF16>
__global__ __launch_bounds__(kQThreads) void quantize_mxfp4_kernel(const void *__restrict__ w, int rows, int cols,
                                                                   uint8_t *__restrict__ q, uint8_t *__restrict__ scales)
{
    const int e = blockIdx.y;
    const int64_t per_expert = (int64_t)rows * cols;
    const int kblocks = cols >> 6, kgroups = (cols + 511) >> 9;
    const int64_t q_expert = per_expert / 2, s_expert = (int64_t)(rows >> 5) * kgroups * 512;
    // eight elements of one row per thread and step; four neighbouring lanes hold one 32-element block.
    // per_expert is a multiple of 2048 (32 rows x 64 columns), so whole waves stay inside the range.
    for (int64_t i = ((int64_t)blockIdx.x * kQThreads + threadIdx.x) * 8; i < per_expert;
         i += (int64_t)gridDim.x * kQThreads * 8) {
        float v[8];
        load4<BF16>(w, (int64_t)e * per_expert + i, *reinterpret_cast<float(*)[4]>(&v[0]));
        load4<BF16>(w, (int64_t)e * per_expert + i + 4, *reinterpret_cast<float(*)[4]>(&v[4]));
        float m = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) m = fmaxf(m, fabsf(v[j]));
        m = fmaxf(m, __shfl_xor(m, 1, 64));
        m = fmaxf(m, __shfl_xor(m, 2, 64));
        // smallest n with m <= 6 * 2^n: m = mant * 2^ex, mant in [0.5, 1), 6 = 0.75 * 2^3
        int n = 0;
        if (m > 0.f) {
            int ex;
            const float mant = frexpf(m, &ex);
            n = mant <= 0.75f ? ex - 3 : ex - 2;
            n = n < -126 ? -126 : n;
        }
        const float inv = ldexpf(1.f, -n);  // exact
        uint32_t word = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) word |= e2m1_code(v[j] * inv) << (4 * j);
        const int64_t r = i / cols;
        const int k = (int)(i - r * cols);
        *reinterpret_cast<uint32_t *>(q + e * q_expert + ((r >> 5) * kblocks + (k >> 6)) * 1024 + (r & 31) * 32 +
                                      ((k & 63) >> 1)) = word;
        if ((k & 31) == 0)
            scales[e * s_expert + ((r >> 5) * kgroups + (k >> 9)) * 512 + (r & 31) * 16 + ((k & 511) >> 5)] =
                (uint8_t)(n + 127);
    }
}

int launch_quantize_mxfp4(int dtype, const void *w, int E, int rows, int cols, uint8_t *q, uint8_t *scales, hipStream_t s)
{
    const int64_t per_expert = (int64_t)rows * cols;
    int64_t bx = (per_expert / 8 + kQThreads * 4 - 1) / (kQThreads * 4);
    if (bx > 512) bx = 512;
    if (bx < 1) bx = 1;
    const dim3 grid((unsigned)bx, (unsigned)E);
    if (dtype == MOE_DTYPE_BF16)
        hipLaunchKernelGGL(quantize_mxfp4_kernel<true>, grid, dim3(kQThreads), 0, s, w, rows, cols, q, scales);
    else
        hipLaunchKernelGGL(quantize_mxfp4_kernel<false>, grid, dim3(kQThreads), 0, s, w, rows, cols, q, scales);
    MOE_LAUNCH_CHECK("quantize_mxfp4");
    return MOE_OK;
}

int launch_quantize_e4m3(int dtype, const void *w, int E, int rows, int cols, uint8_t *q, float *scale, hipStream_t s)
{
    const int64_t per_expert = (int64_t)rows * cols;
    uint32_t *bits = reinterpret_cast<uint32_t *>(scale);
    int rc = launch_fill_u32(bits, E, 0u, s);
    if (rc != MOE_OK) return rc;
    int64_t bx = (per_expert + (int64_t)kQThreads * 16 - 1) / ((int64_t)kQThreads * 16);
    if (bx > 256) bx = 256;
    if (bx < 1) bx = 1;
    const dim3 grid((unsigned)bx, (unsigned)E);
    if (dtype == MOE_DTYPE_BF16) {
        hipLaunchKernelGGL(absmax_kernel<true>, grid, dim3(kQThreads), 0, s, w, per_expert, bits);
        hipLaunchKernelGGL(quantize_kernel<true>, grid, dim3(kQThreads), 0, s, w, per_expert, cols, bits, q);
    } else {
        hipLaunchKernelGGL(absmax_kernel<false>, grid, dim3(kQThreads), 0, s, w, per_expert, bits);
        hipLaunchKernelGGL(quantize_kernel<false>, grid, dim3(kQThreads), 0, s, w, per_expert, cols, bits, q);
    }
    hipLaunchKernelGGL(finish_scale_kernel, dim3(ceil_div(E, 256)), dim3(256), 0, s, bits, E);
    MOE_LAUNCH_CHECK("quantize_e4m3");
    return MOE_OK;
}

}  // namespace moe355
