// Internal declarations shared by the HIP translation units of libmoe355.
// Nothing here is part of the C ABI (include/moe.h is).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe.h"

namespace moe355 {
// Optional per-kernel timing with HIP events recorded on the stream the kernels run on.
struct Profiler {
    static constexpr int kMax = 64;
    bool enabled = false;
    int n = 0;
    const char *names[kMax];
    hipEvent_t start[kMax];
    hipEvent_t stop[kMax];
    int created = 0;  // events [0, created) exist
};

// ---- static-capacity baseline (static_baseline.hip) ---------------------------------------------
// idx [T,k] -> idx_t [k*T] (slot-major: all first choices, then all second choices, ...); also
// clears dropped[0].
int launch_transpose_idx(const int32_t *idx, int T, int k, int32_t *idx_t, int32_t *dropped, hipStream_t s);
// pos [k*T] = offsets_s[e] + rank of the assignment inside expert e in slot-major order (from the
// routing kernels run on idx_t).  slot_row[t,j] = e*capacity + slot, or -1 when slot >= capacity;
// dropped[0] += number of -1.
int launch_static_rows(const int32_t *idx_t, const int32_t *pos, const int32_t *offsets_s, int T, int k, int E,
                       int capacity, int32_t *slot_row, int32_t *dropped, hipStream_t s);
int launch_fill_u32(void *dst, int64_t n_words, uint32_t value, hipStream_t s);
// row_tok[slot_row[t,j]] = t for kept assignments (row_tok pre-filled with -1)
int launch_row_tokens(const int32_t *slot_row, int T, int k, int32_t *row_tok, hipStream_t s);
// xd[r,:] = row_tok[r] >= 0 ? x[row_tok[r],:] : 0     (rows = E*capacity)
int launch_padded_gather(int dtype, const void *x, const int32_t *row_tok, int64_t rows, int D, void *xd,
                         hipStream_t s);
// offsets_static[e] = e*capacity, e = 0..E
int launch_static_offsets(int32_t *offsets_static, int E, int capacity, hipStream_t s);
// out [C, ldo] = in[R, C]^T, columns R..ldo-1 zero     (element size 2 or 4 bytes)
int launch_transpose_pad(int dtype, const void *in, int64_t R, int64_t C, void *out, int64_t ldo, hipStream_t s);
// one-hot dispatch mask: mask[slot_row[t,j], t] = 1 (elem), ld = ldm;  combine weights:
// cw[t, slot_row[t,j]] = w[t,j] (elem), ld = ldc.  Both pre-zeroed.
int launch_static_masks(int dtype, const int32_t *slot_row, const float *w, int T, int k, void *mask, int64_t ldm,
                        void *cw, int64_t ldc, hipStream_t s);

}  // namespace moe355

struct moe_handle {
    moe_config_t cfg;
    int device;
    int num_cus;
    void *scratch;  // device address of the library's own scratch array on `device` (moe_layer_forward_noalloc)
    moe355::Profiler prof;
};

struct moe_cache_policy;

namespace moe355 {

// ---- errors -----------------------------------------------------------------------------------
void set_error(const char *fmt, ...);
int hip_failed(hipError_t e, const char *what);  // records the message, returns MOE_ERR_HIP
#define MOE_HIP_CHECK(expr)                                                  \
    do {                                                                     \
        hipError_t _e = (expr);                                              \
        if (_e != hipSuccess) return ::moe355::hip_failed(_e, #expr);        \
    } while (0)
#define MOE_LAUNCH_CHECK(name)                                               \
    do {                                                                     \
        hipError_t _e = hipGetLastError();                                   \
        if (_e != hipSuccess) return ::moe355::hip_failed(_e, name);         \
    } while (0)

// Brackets one kernel launch with events when the calling entry point's handle has profiling on.
struct ProfScope {
    ProfScope(const char *name, hipStream_t s);
    ~ProfScope();
    hipStream_t stream;
    int slot;
};
// Binds the handle's profiler to the calling thread for the duration of an entry point.
struct ProfBind {
    explicit ProfBind(moe_handle *h);
    ~ProfBind();
};

__host__ __device__ static inline int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }
__host__ __device__ static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// ---- grouped / plain GEMM  C = A * B^T  (both operands K-contiguous) ---------------------------
// Plain mode: one problem of M rows.  Grouped mode: rows [offsets[e], offsets[e+1]) of A use
// B + e*strideB; M tiles never straddle two experts (the tile map says which expert and which
// first row every M tile has).
struct GemmParams {
    const void *A;       // [rows, K]
    int64_t lda;
    const int32_t *a_rows;  // bf16 grouped kernels: logical row r of A is row a_rows[r] of the array (NULL = r)
    const void *B;       // [N, K] (plain) or [E, N, K] (grouped)
    int64_t ldb;
    int64_t strideB;     // elements between experts (between slots with b_slot)
    const int32_t *b_slot;  // grouped: expert e's weights are slot b_slot[e] of B (NULL = e)
    const float *b_scale;   // 8-bit weight variants: fp32 scale per expert (NULL = 1)
    const uint8_t *b_blk_scale;  // 4-bit weight variants: e8m0 scale bytes, per expert [N/32][ceil(K/512)][32][16]
    int64_t stride_blk_scale;    // bytes between two experts' scale arrays
    const void *bias;    // elem [N] / [E,N], or NULL
    int64_t strideBias;
    const float *bias_f32;  // fp32 [N] or NULL (gate offsets)
    void *C;             // [rows, N]
    int64_t ldc;
    int M, N, K;
    // plain mode, fp32 C: K cut into k_split ranges (0 / 1 = whole K); range 0 writes C, range i > 0 writes
    // c_parts + (i - 1) * split_stride (same ldc)
    int k_split;
    int64_t split_stride;
    float *c_parts;
    // grouped mode
    const int32_t *offsets;      // [E+1]
    const int32_t *tile_expert;  // [max_m_tiles]
    const int32_t *tile_row;     // [max_m_tiles] first row of the tile
    const int32_t *num_tiles;    // [1]
    int max_m_tiles;             // host upper bound of *num_tiles (sizes the grid)
    // tail splitting of a grouped GEMM over 256x256 tiles (0 = off): 1 = this launch runs the whole
    // rounds of 256x256 tiles, 2 = this launch runs the tiles of the last, partly filled round as
    // smaller sub-tiles; main_slots = grid size of the launch with tail_mode 1 (both need it)
    int tail_mode;
    int main_slots;
    // grouped bf16 kernels.  a_zero_row >= 0: row of A's array that is all zero; tile rows past the end of an
    // expert's batch read it instead of repeating the batch's last row (their results are discarded either way,
    // but zeros cost the matrix pipes less power than live data, and the clock is power-limited).
    // c_zero_row >= 0: the launch also writes zeros to that row of C (the next GEMM's a_zero_row).
    int a_zero_row;
    int c_zero_row;
    const char *name;            // host only: label of the launch for the event profiler (may be NULL)
};

// Tile shape (an opaque variant id) the grouped GEMM uses for n_rows rows over E experts and N
// output columns, and the M tile height of a variant; the tile map must be built with that height.
int gemm_variant(int dtype, int64_t n_rows, int E, int N, int num_cus);
int gemm_variant_block_m(int dtype, int variant);
// true when the variant's kernel can read its A rows through GemmParams::a_rows
bool gemm_variant_gathers(int dtype, int variant);

// variant: from gemm_variant (grouped) or 0 (plain).  out_f32: C is fp32 (else elem); relu:
// max(.,0) before the store.
int launch_gemm(int dtype, const GemmParams &p, bool grouped, int variant, bool out_f32, bool relu,
                int num_cus, hipStream_t s);

// 8-bit weights (quant.hip): q [E, per_expert] e4m3 bytes and scale [E] from w [E, per_expert] (dtype elem);
// per_expert a multiple of 4.
int launch_quantize_e4m3(int dtype, const void *w, int E, int rows, int cols, uint8_t *q, float *scale,
                         hipStream_t s);
int launch_quantize_mxfp4(int dtype, const void *w, int E, int rows, int cols, uint8_t *q, uint8_t *scales,
                          hipStream_t s);

// Tile map for the grouped GEMM from the device-side offsets (one block).
// stage_of != NULL: only the experts e with stage_of[e] == stage get tiles.
int launch_tile_map(const int32_t *offsets, int E, int block_m, int32_t *tile_expert, int32_t *tile_row,
                    int32_t *num_tiles, int max_m_tiles, const int32_t *stage_of, int stage, hipStream_t s);

// ---- routing -------------------------------------------------------------------------------------
int launch_topk(float *logits, int T, int E, int k, int renorm, int32_t *idx, float *w, hipStream_t s, int n_parts = 1,
                const float *parts = nullptr, int64_t part_stride = 0);
// block_hist: scratch of route_blocks(T)*E int32
int route_blocks(int T);
// true when launch_route for T tokens with k experts each reads per-block histograms (large batches); small
// ones are routed by one block that needs none
bool route_uses_hist(int T, int k);
// hist_tokens > 0: block_hist already holds one histogram row per hist_tokens tokens (a divisor of 256)
int launch_route(const int32_t *idx, int T, int E, int k, int32_t *counts, int32_t *offsets, int32_t *dst_row,
                 int32_t *src_tok, int32_t *block_hist, hipStream_t s, int tile_bm = 0, int32_t *tile_expert = nullptr,
                 int32_t *tile_row = nullptr, int32_t *num_tiles = nullptr, int max_m_tiles = 0, int hist_tokens = 0);

// Gate GEMM with softmax / top-k and the per-tile expert histogram in its epilogue (gate_topk.hip); bf16, E <= 128,
// K a multiple of 64.  logits and hist may be NULL.  hist gets one row per gate_topk_tile_tokens() tokens.
bool gate_topk_fused_ok(int dtype, int T, int E, int K);
int gate_topk_tile_tokens(int T, int E, int num_cus);
int launch_gate_topk(const void *x, const void *wg, const float *gate_bias, int T, int E, int K, int k, int renorm,
                     float *logits, int32_t *idx, float *w, int32_t *hist, int num_cus, hipStream_t s);

// ---- row movement --------------------------------------------------------------------------------
int launch_dispatch(int dtype, const void *x, const int32_t *dst_row, int T, int D, int k, void *xp,
                    hipStream_t s);
int launch_combine(int dtype, const void *yp, const int32_t *dst_row, const float *w, int T, int D, int k,
                   void *y, hipStream_t s);

}  // namespace moe355
