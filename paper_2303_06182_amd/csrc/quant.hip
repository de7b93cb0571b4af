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
