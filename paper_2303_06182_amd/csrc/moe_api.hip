// C-ABI entry points of libmoe355 (declared in include/moe.h): argument validation on the host,
// workspace carving, and the launch sequences.  No entry point allocates device memory, waits
// for the device, or reads device data on the host.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "moe_internal.h"

namespace moe355 {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int hip_failed(hipError_t e, const char *what)
{
    set_error("HIP error %d (%s) at %s", (int)e, hipGetErrorString(e), what);
    return MOE_ERR_HIP;
}

// ---- scratch for the entry point that allocates nothing -------------------------------------------
// moe_layer_forward_noalloc carves its workspace out of this array instead of a caller buffer.  Every
// device the library runs on holds its own copy at its own address until the process ends.  On the
// host the array's name is only a handle for hipGetSymbolAddress: the address that kernels, copies
// and fills get is the one that call returned for the current device (scratch_for_device), never
// the name.
static __device__ __align__(256) __attribute__((used)) uint8_t scratch[MOE_NOALLOC_SCRATCH_BYTES];

static constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices];  // per device ordinal; NULL = not looked up yet

// Address of `scratch` on device `dev`, which must be the current device.  Looked up once per device.
static int scratch_for_device(int dev, void **out)
{
    *out = nullptr;
    if (dev < 0 || dev >= kMaxDevices) {
        set_error("device ordinal %d outside [0, %d)", dev, kMaxDevices);
        return MOE_ERR_INVALID_ARG;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        MOE_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || reinterpret_cast<uintptr_t>(ptr) % 256 != 0) {
            set_error("the library's scratch array has no usable device address");
            return MOE_ERR_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return MOE_OK;
}

// ---- per-kernel event timing ---------------------------------------------------------------------
static thread_local Profiler *g_prof = nullptr;

ProfBind::ProfBind(moe_handle *h) { g_prof = (h && h->prof.enabled) ? &h->prof : nullptr; }
ProfBind::~ProfBind() { g_prof = nullptr; }

ProfScope::ProfScope(const char *name, hipStream_t s) : stream(s), slot(-1)
{
    Profiler *p = g_prof;
    if (!p || p->n >= Profiler::kMax) return;
    while (p->created <= p->n) {
        if (hipEventCreate(&p->start[p->created]) != hipSuccess) return;
        if (hipEventCreate(&p->stop[p->created]) != hipSuccess) {
            (void)hipEventDestroy(p->start[p->created]);
            return;
        }
        p->created += 1;
    }
    slot = p->n++;
    p->names[slot] = name;
    (void)hipEventRecord(p->start[slot], stream);
}

ProfScope::~ProfScope()
{
    if (slot >= 0 && g_prof) (void)hipEventRecord(g_prof->stop[slot], stream);
}

int launch_gemm_bf16(const GemmParams &p, bool grouped, int variant, bool out_f32, bool relu, int num_cus,
                     hipStream_t s);
int gemm_bf16_variant(int64_t n_rows, int E, int N, int num_cus);
int gemm_bf16_variant_block_m(int variant);
int launch_gemm_f32(const GemmParams &p, bool grouped, bool relu, hipStream_t s);
int gemm_f32_block_m();
bool gemm_bf16_variant_gathers(int variant, int K);
int gemm_bf16_variant_w8(int64_t n_rows, int E);
int gemm_bf16_variant_w4(int64_t n_rows, int E);
int gemm_bf16_gate_split(int M, int N, int K, int num_cus);

int gemm_variant(int dtype, int64_t n_rows, int E, int N, int num_cus)
{
    return dtype == MOE_DTYPE_BF16 ? gemm_bf16_variant(n_rows, E, N, num_cus) : 0;
}

int gemm_variant_block_m(int dtype, int variant)
{
    return dtype == MOE_DTYPE_BF16 ? gemm_bf16_variant_block_m(variant) : gemm_f32_block_m();
}

int launch_gemm(int dtype, const GemmParams &p, bool grouped, int variant, bool out_f32, bool relu, int num_cus,
                hipStream_t s)
{
    ProfScope ps(p.name ? p.name : (!grouped ? "gate_gemm" : (relu ? "expert_gemm1" : "expert_gemm2")), s);
    if (dtype == MOE_DTYPE_BF16) return launch_gemm_bf16(p, grouped, variant, out_f32, relu, num_cus, s);
    return launch_gemm_f32(p, grouped, relu, s);  // fp32 storage: C is fp32 either way
}

// ---- workspace ---------------------------------------------------------------------------------
static constexpr int kMinBlockM = 32;  // smallest M tile any grouped GEMM uses: sizes the tile map
// split K of the gate GEMM: at most this many K ranges, only for this many tokens or fewer (sizes the slices)
static constexpr int kGateSplitMax = 16, kGateSplitTokens = 256;

struct WsLayout {
    int64_t logits, topk_idx, topk_w, counts, offsets, dst_row, src_tok, block_hist;
    int64_t tile_expert, tile_row, num_tiles, gate_parts, xp, h, yp, total;
};

static int elem_size(int dtype) { return dtype == MOE_DTYPE_BF16 ? 2 : 4; }

static WsLayout ws_layout(const moe_config_t &c)
{
    WsLayout L;
    const int64_t T = c.T_max, N = (int64_t)c.T_max * c.k, E = c.E, es = elem_size(c.dtype);
    int64_t off = 0;
    auto take = [&](int64_t bytes) {
        const int64_t at = off;
        off = align_up(off + (bytes > 0 ? bytes : 1), 256);
        return at;
    };
    L.logits = take(T * E * 4);
    L.topk_idx = take(N * 4);
    L.topk_w = take(N * 4);
    L.counts = take(E * 4);
    L.offsets = take((E + 1) * 4);
    L.dst_row = take(N * 4);
    L.src_tok = take(N * 4);
    // one histogram row per 256 tokens (routing step) or per tile of the fused gate kernel (32 tokens at least)
    L.block_hist = take(((T + 31) / 32 > route_blocks((int)T) ? (T + 31) / 32 : route_blocks((int)T)) * E * 4);
    const int64_t max_tiles = N / kMinBlockM + E + 1;
    L.tile_expert = take(max_tiles * 4);
    L.tile_row = take(max_tiles * 4);
    L.num_tiles = take(4);
    L.gate_parts = take((int64_t)(kGateSplitMax - 1) * (T < kGateSplitTokens ? T : kGateSplitTokens) * E * 4);
    L.xp = take(N * c.D * es);
    L.h = take((N + 1) * c.F * es);  // one more row: zeros, read for the padded rows of the second GEMM's tiles
    L.yp = take(N * c.D * es);
    L.total = off;
    return L;
}

template <typename T>
static T *at(void *ws, int64_t off)
{
    return reinterpret_cast<T *>(static_cast<uint8_t *>(ws) + off);
}

// ---- validation --------------------------------------------------------------------------------
static bool bad_ptr(const void *p, const char *name, bool nullable = false)
{
    if (!p) {
        if (nullable) return false;
        set_error("%s is NULL", name);
        return true;
    }
    if (reinterpret_cast<uintptr_t>(p) % 16 != 0) {
        set_error("%s is not 16-byte aligned", name);
        return true;
    }
    return false;
}

static int check_handle_T(const moe_handle_t *h, int32_t T)
{
    if (!h) {
        set_error("handle is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    if (T < 0 || T > h->cfg.T_max) {
        set_error("T = %d outside [0, T_max = %d]", T, h->cfg.T_max);
        return MOE_ERR_INVALID_ARG;
    }
    return MOE_OK;
}

static int check_ws(const moe_handle_t *h, const void *ws, int64_t bytes)
{
    if (!ws) {
        set_error("workspace is NULL");
        return MOE_ERR_WORKSPACE;
    }
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) {
        set_error("workspace is not 256-byte aligned");
        return MOE_ERR_WORKSPACE;
    }
    const int64_t need = ws_layout(h->cfg).total;
    if (bytes < need) {
        set_error("workspace has %lld bytes, %lld needed", (long long)bytes, (long long)need);
        return MOE_ERR_WORKSPACE;
    }
    return MOE_OK;
}

static int validate_config(const moe_config_t *c)
{
    if (!c) {
        set_error("config is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    if (c->dtype != MOE_DTYPE_F32 && c->dtype != MOE_DTYPE_BF16) {
        set_error("unsupported dtype %d", c->dtype);
        return MOE_ERR_UNSUPPORTED;
    }
    if (c->E < 1 || c->E > MOE_MAX_E) {
        set_error("E = %d outside [1, %d]", c->E, MOE_MAX_E);
        return MOE_ERR_UNSUPPORTED;
    }
    if (c->k < 1 || c->k > MOE_MAX_K || c->k > c->E) {
        set_error("k = %d outside [1, min(E, %d)]", c->k, MOE_MAX_K);
        return MOE_ERR_UNSUPPORTED;
    }
    if (c->D < 8 || c->D % 8 != 0 || c->F < 8 || c->F % 8 != 0) {
        set_error("D = %d and F = %d must be positive multiples of 8", c->D, c->F);
        return MOE_ERR_UNSUPPORTED;
    }
    if (c->T_max < 0) {
        set_error("T_max = %d is negative", c->T_max);
        return MOE_ERR_INVALID_ARG;
    }
    if ((int64_t)c->T_max * c->k > 0x3fffffff) {
        set_error("k * T_max = %lld does not fit the int32 row indices", (long long)c->T_max * c->k);
        return MOE_ERR_INVALID_ARG;
    }
    if (c->renormalize != 0 && c->renormalize != 1) {
        set_error("renormalize must be 0 or 1");
        return MOE_ERR_INVALID_ARG;
    }
    return MOE_OK;
}

// ---- the five steps ------------------------------------------------------------------------------
// logits_req: where the caller wants the [T,E] logits, or NULL; logits_ws: room for them in the workspace, used
// when a kernel needs them in memory and the caller did not ask (NULL only together with a non-NULL logits_req).
// parts: room for (kGateSplitMax - 1) * min(T_max, kGateSplitTokens) * E floats, or NULL.  A decoder step's
// gate GEMM (a tile or two, a long K loop) is cut along K into slices that the top-k kernel adds up.
// hist != NULL: a kernel that decides the routing in the gate GEMM's epilogue may also leave the per-tile expert
// histogram there (room for ceil(T / 32) * E int32); *hist_tokens then says how many tokens one row covers (0 =
// no histogram was written and the routing step makes its own).
static int do_gate_topk(moe_handle_t *h, const void *x, const void *wg, const float *gate_bias, int T,
                        float *logits_req, float *logits_ws, int32_t *idx, float *w, hipStream_t s,
                        float *parts = nullptr, int32_t *hist = nullptr, int *hist_tokens = nullptr)
{
    const moe_config_t &c = h->cfg;
    if (hist_tokens) *hist_tokens = 0;
    if (T == 0) return MOE_OK;
    // Batches beyond a decoder step, bf16, at most 128 experts: one kernel streams x, keeps the logits in
    // registers and writes the decision (and the logits only where the caller asked for them).
    if (T > kGateSplitTokens && gate_topk_fused_ok(c.dtype, T, c.E, c.D)) {
        const bool want_hist = hist && hist_tokens && route_uses_hist(T, c.k);
        int rc = launch_gate_topk(x, wg, gate_bias, T, c.E, c.D, c.k, c.renormalize, logits_req, idx, w,
                                  want_hist ? hist : nullptr, h->num_cus, s);
        if (rc == MOE_OK && want_hist) *hist_tokens = gate_topk_tile_tokens(T, c.E, h->num_cus);
        return rc;
    }
    float *logits = logits_req ? logits_req : logits_ws;
    int split = 1;
    if (parts && c.dtype == MOE_DTYPE_BF16 && T <= kGateSplitTokens) {
        split = gemm_bf16_gate_split(T, c.E, c.D, h->num_cus);
        if (split > kGateSplitMax) split = kGateSplitMax;
    }
    GemmParams p;
    memset(&p, 0, sizeof(p));
    p.A = x;
    p.lda = c.D;
    p.B = wg;
    p.ldb = c.D;
    p.bias_f32 = gate_bias;
    p.C = logits;
    p.ldc = c.E;
    p.M = T;
    p.N = c.E;
    p.K = c.D;
    if (split > 1) {
        p.k_split = split;
        p.c_parts = parts;
        p.split_stride = (int64_t)T * c.E;
    }
    int rc = launch_gemm(c.dtype, p, false, 0, true, false, h->num_cus, s);
    if (rc != MOE_OK) return rc;
    return launch_topk(logits, T, c.E, c.k, c.renormalize, idx, w, s, split, parts, p.split_stride);
}

// scale bytes of one expert's [rows, cols] matrix in the 4-bit layout: 16 per row and 512 columns
static int64_t mxfp4_scale_bytes(int64_t rows, int64_t cols) { return (rows / 32) * ((cols + 511) / 512) * 512; }

// tile shape of the grouped GEMM for quantised weights
static int quant_variant(int wbits, int64_t n_rows, int E)
{
    return wbits == 4 ? gemm_bf16_variant_w4(n_rows, E) : gemm_bf16_variant_w8(n_rows, E);
}

// Options of the grouped FFN beyond the plain call.
struct FfnExtra {
    // xp is the token array and row r of the experts' input is its row a_rows[r] (dispatch fused
    // into the first GEMM's loads; the caller checked fused_dispatch_ok)
    const int32_t *a_rows = nullptr;
    // expert buffering: w1 / w2 point at the first slot's W1 / W2, slots are slot_stride elements
    // apart, expert e's weights are in slot b_slot[e], and only experts with stage_of[e] == stage run
    const int32_t *b_slot = nullptr;
    const int32_t *stage_of = nullptr;
    int stage = 0;
    int64_t slot_stride = 0;
    // the routing step has already written the tile map for M tiles of this height (0 = it has not)
    int tile_map_ready_bm = 0;
    // 8-bit weights: w1 / w2 are e4m3 bytes, one fp32 scale per expert and matrix
    const float *w1_scale = nullptr;     // 8-bit weights: per-expert scales
    const float *w2_scale = nullptr;
    const uint8_t *w1_blk = nullptr;     // 4-bit weights: block scale bytes
    const uint8_t *w2_blk = nullptr;
};

// Grouped FFN on n_rows rows split by offsets[]; hbuf [n_rows + 1, F] and the tile arrays are scratch.
static int run_expert_ffn(moe_handle_t *h, const void *xp, const FfnExtra &ex, const int32_t *offsets,
                          const void *w1, const void *w2, const void *b1, const void *b2, int64_t n_rows, void *yp,
                          void *hbuf, int32_t *tile_expert, int32_t *tile_row, int32_t *num_tiles, hipStream_t s)
{
    const moe_config_t &c = h->cfg;
    if (n_rows == 0) return MOE_OK;
    // each GEMM picks its own tile shape (N differs: F for the first, D for the second); the tile
    // map is rebuilt between them only when the M tile height differs
    const int wbits = ex.w1_blk ? 4 : ex.w1_scale ? 8 : 0;
    const int v1 = wbits ? quant_variant(wbits, n_rows, c.E) : gemm_variant(c.dtype, n_rows, c.E, c.F, h->num_cus);
    const int v2 = wbits ? v1 : gemm_variant(c.dtype, n_rows, c.E, c.D, h->num_cus);
    const int bm1 = gemm_variant_block_m(c.dtype, v1), bm2 = gemm_variant_block_m(c.dtype, v2);
    int max_tiles = (int)(n_rows / bm1) + c.E + 1;
    int rc = MOE_OK;
    if (ex.stage_of || ex.tile_map_ready_bm != bm1) {
        rc = launch_tile_map(offsets, c.E, bm1, tile_expert, tile_row, num_tiles, max_tiles, ex.stage_of, ex.stage, s);
        if (rc != MOE_OK) return rc;
    }

    GemmParams p;
    memset(&p, 0, sizeof(p));
    p.offsets = offsets;
    p.tile_expert = tile_expert;
    p.tile_row = tile_row;
    p.num_tiles = num_tiles;
    p.max_m_tiles = max_tiles;
    p.M = (int)n_rows;
    p.a_zero_row = -1;
    // The first GEMM leaves a zero row behind H's n_rows rows (hbuf has room for it); the second reads it for the
    // rows of a tile that lie past the end of an expert's batch.  (Row offsets inside the kernel are 32-bit.)
    const bool zero_row = c.dtype == MOE_DTYPE_BF16 && (n_rows + 1) * (int64_t)c.F < ((int64_t)1 << 31);
    p.c_zero_row = zero_row ? (int)n_rows : -1;
    // H = relu(Xp * W1[e]^T + b1[e])
    p.A = xp;
    p.a_rows = ex.a_rows;
    p.lda = c.D;
    p.B = w1;
    p.b_slot = ex.b_slot;
    p.b_scale = ex.w1_scale;
    p.ldb = c.D;
    p.strideB = ex.b_slot ? ex.slot_stride : (int64_t)c.F * c.D / (wbits == 4 ? 2 : 1);  // elements; bytes for 8 and 4 bits
    p.b_blk_scale = ex.w1_blk;
    p.stride_blk_scale = mxfp4_scale_bytes(c.F, c.D);
    p.bias = b1;
    p.strideBias = c.F;
    p.C = hbuf;
    p.ldc = c.F;
    p.N = c.F;
    p.K = c.D;
    rc = launch_gemm(c.dtype, p, true, v1, false, true, h->num_cus, s);
    if (rc != MOE_OK) return rc;
    if (bm2 != bm1) {
        max_tiles = (int)(n_rows / bm2) + c.E + 1;
        rc = launch_tile_map(offsets, c.E, bm2, tile_expert, tile_row, num_tiles, max_tiles, ex.stage_of, ex.stage, s);
        if (rc != MOE_OK) return rc;
        p.max_m_tiles = max_tiles;
    }
    // Yp = H * W2[e]^T + b2[e]
    p.A = hbuf;
    p.a_rows = nullptr;
    p.a_zero_row = zero_row ? (int)n_rows : -1;
    p.c_zero_row = -1;
    p.lda = c.F;
    p.B = w2;
    p.b_scale = ex.w2_scale;
    p.ldb = c.F;
    p.strideB = ex.b_slot ? ex.slot_stride : (int64_t)c.D * c.F / (wbits == 4 ? 2 : 1);
    p.b_blk_scale = ex.w2_blk;
    p.stride_blk_scale = mxfp4_scale_bytes(c.D, c.F);
    p.bias = b2;
    p.strideBias = c.D;
    p.C = yp;
    p.ldc = c.D;
    p.N = c.D;
    p.K = c.F;
    return launch_gemm(c.dtype, p, true, v2, false, false, h->num_cus, s);
}

// Can the first expert GEMM gather its rows from the token array (T tokens) itself?
static bool fused_dispatch_ok(const moe_handle_t *h, int64_t T, int wbits = 0)
{
    const moe_config_t &c = h->cfg;
    if (c.dtype != MOE_DTYPE_BF16 || T * c.D >= ((int64_t)1 << 31)) return false;
    const int v = wbits ? quant_variant(wbits, T * c.k, c.E) : gemm_variant(c.dtype, T * c.k, c.E, c.F, h->num_cus);
    return gemm_bf16_variant_gathers(v, c.D);
}

// 8- and 4-bit weights need bf16 activations and K dimensions that are whole K tiles
static int check_w8(const moe_handle_t *h)
{
    const moe_config_t &c = h->cfg;
    if (c.dtype != MOE_DTYPE_BF16 || c.D % 64 != 0 || c.F % 64 != 0) {
        set_error("8- and 4-bit expert weights need dtype bf16 and D, F multiples of 64 (D = %d, F = %d)", c.D, c.F);
        return MOE_ERR_UNSUPPORTED;
    }
    return MOE_OK;
}

static int do_expert_ffn(moe_handle_t *h, const void *xp, const FfnExtra &ex, const int32_t *offsets,
                         const void *w1, const void *w2, const void *b1, const void *b2, int n_rows, void *yp,
                         void *ws, hipStream_t s)
{
    const WsLayout L = ws_layout(h->cfg);
    return run_expert_ffn(h, xp, ex, offsets, w1, w2, b1, b2, n_rows, yp, at<void>(ws, L.h),
                          at<int32_t>(ws, L.tile_expert), at<int32_t>(ws, L.tile_row), at<int32_t>(ws, L.num_tiles), s);
}

// ---- static-capacity baseline --------------------------------------------------------------------
struct StaticLayout {
    int64_t logits, topk_idx, topk_w, idx_t, counts_s, offsets_s, pos, src_s, block_hist, slot_row, row_tok;
    int64_t offsets_static, tile_expert, tile_row, num_tiles, xd, hd, yd, xt, ydt, mask, cw, total;
    int64_t ldt, ldk;  // padded leading dimensions (elements) of the T-long and E*cap-long K axes
};

static StaticLayout static_layout(const moe_config_t &c, int64_t T, int64_t cap, int mode)
{
    StaticLayout L;
    memset(&L, 0, sizeof(L));
    const int64_t N = T * c.k, E = c.E, es = elem_size(c.dtype), R = E * cap;
    int64_t off = 0;
    auto take = [&](int64_t bytes) {
        const int64_t at = off;
        off = align_up(off + (bytes > 0 ? bytes : 1), 256);
        return at;
    };
    L.ldt = align_up(T, 64);
    L.ldk = align_up(R, 64);
    L.logits = take(T * E * 4);
    L.topk_idx = take(N * 4);
    L.topk_w = take(N * 4);
    L.idx_t = take(N * 4);
    L.counts_s = take(E * 4);
    L.offsets_s = take((E + 1) * 4);
    L.pos = take(N * 4);
    L.src_s = take(N * 4);
    L.block_hist = take((int64_t)route_blocks((int)N) * E * 4);
    L.slot_row = take(N * 4);
    L.row_tok = take(R * 4);
    L.offsets_static = take((E + 1) * 4);
    const int64_t max_tiles = R / kMinBlockM + E + 1;
    L.tile_expert = take(max_tiles * 4);
    L.tile_row = take(max_tiles * 4);
    L.num_tiles = take(4);
    L.xd = take(R * c.D * es);
    L.hd = take((R + 1) * c.F * es);
    L.yd = take(R * c.D * es);
    if (mode == MOE_STATIC_EINSUM) {
        L.xt = take((int64_t)c.D * L.ldt * es);
        L.ydt = take((int64_t)c.D * L.ldk * es);
        L.mask = take(R * L.ldt * es);
        L.cw = take(T * L.ldk * es);
    }
    L.total = off;
    return L;
}

// ---- expert buffering (paper Sec. 6) ----------------------------------------------------------
int cache_policy_step(moe_cache_policy *p, const int32_t *counts, int32_t *slot_of, int32_t *stage_of,
                      int32_t *loads, int32_t max_loads, int32_t *n_loads, int32_t *n_stages);

}  // namespace moe355

struct moe_expert_cache {
    moe_handle_t *h = nullptr;
    moe_cache_policy_t *policy = nullptr;
    int slots = 0;
    const uint8_t *host_w1 = nullptr, *host_w2 = nullptr;
    int64_t half_bytes = 0;        // one expert's W1 (= W2) in bytes
    int wbits = 0;                 // 0: elem weights; 8 / 4: e4m3 bytes / e2m1 nibbles in the host arrays and slots
    const void *scale1 = nullptr, *scale2 = nullptr;  // device, all experts: fp32 [E] (8) or block scale bytes (4)
    uint8_t *d_slots = nullptr;    // [slots][W1 | W2]
    int32_t *d_slot_of = nullptr;  // [E] slot an active expert runs from
    int32_t *d_stage = nullptr;    // [E] launch it runs in (2 * stage + missed), -1 idle
    int32_t *pin = nullptr;        // pinned host: counts[E] | slot_of[E] | launch stage[E]
    hipStream_t copy_stream = nullptr;
    std::vector<hipEvent_t> events;  // grown on demand, reused by every call
    std::vector<int32_t> stage_of, loads;
    int64_t bytes_copied = 0, stages = 0;
};

namespace moe355 {

static int64_t cache_index_bytes(const moe_config_t &c) { return align_up((int64_t)c.E * 4, 256); }

static int cache_event(moe_expert_cache *c, size_t i, hipEvent_t *out)
{
    while (c->events.size() <= i) {
        hipEvent_t e;
        MOE_HIP_CHECK(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        c->events.push_back(e);
    }
    *out = c->events[i];
    return MOE_OK;
}

}  // namespace moe355

using namespace moe355;

extern "C" {

const char *moe_last_error(void) { return g_err; }

int moe_create(const moe_config_t *cfg, moe_handle_t **out)
{
    g_err[0] = 0;
    if (!out) {
        set_error("out is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    *out = nullptr;
    int rc = validate_config(cfg);
    if (rc != MOE_OK) return rc;
    int dev = 0;
    MOE_HIP_CHECK(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    MOE_HIP_CHECK(hipGetDeviceProperties(&prop, dev));
    moe_handle_t *h = new (std::nothrow) moe_handle_t;
    if (!h) {
        set_error("out of host memory");
        return MOE_ERR_INVALID_ARG;
    }
    h->cfg = *cfg;
    h->device = dev;
    h->num_cus = prop.multiProcessorCount;
    // the current device is `dev`: the one moment at which its copy of the scratch array can be looked up
    rc = scratch_for_device(dev, &h->scratch);
    if (rc != MOE_OK) {
        delete h;
        return rc;
    }
    *out = h;
    return MOE_OK;
}

int moe_destroy(moe_handle_t *h)
{
    if (h) {
        for (int i = 0; i < h->prof.created; ++i) {
            (void)hipEventDestroy(h->prof.start[i]);
            (void)hipEventDestroy(h->prof.stop[i]);
        }
    }
    delete h;
    return MOE_OK;
}

int moe_profile_begin(moe_handle_t *h)
{
    g_err[0] = 0;
    if (!h) {
        set_error("handle is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    h->prof.enabled = true;
    h->prof.n = 0;
    return MOE_OK;
}

int moe_profile_end(moe_handle_t *h, float *ms_out, int32_t max_records, int32_t *n_records)
{
    g_err[0] = 0;
    if (!h || !n_records || (max_records > 0 && !ms_out)) {
        set_error("moe_profile_end: NULL argument");
        return MOE_ERR_INVALID_ARG;
    }
    Profiler &p = h->prof;
    p.enabled = false;
    const int n = p.n < max_records ? p.n : max_records;
    for (int i = 0; i < n; ++i) {
        MOE_HIP_CHECK(hipEventSynchronize(p.stop[i]));
        MOE_HIP_CHECK(hipEventElapsedTime(&ms_out[i], p.start[i], p.stop[i]));
    }
    *n_records = n;
    return MOE_OK;
}

const char *moe_profile_name(const moe_handle_t *h, int32_t i)
{
    if (!h || i < 0 || i >= h->prof.n) return "";
    return h->prof.names[i];
}

int64_t moe_workspace_bytes(const moe_handle_t *h)
{
    if (!h) {
        set_error("handle is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    return ws_layout(h->cfg).total;
}

int32_t moe_capacity(int32_t T, int32_t E, int32_t k, double cf, int32_t convention)
{
    if (T < 0 || E < 1 || k < 1 || !(cf > 0.0)) {
        set_error("moe_capacity: bad arguments");
        return MOE_ERR_INVALID_ARG;
    }
    double rows;
    if (convention == MOE_CAPACITY_PAPER)
        rows = cf * (double)T;
    else if (convention == MOE_CAPACITY_SHARE)
        rows = cf * (double)k * (double)T / (double)E;
    else {
        set_error("moe_capacity: unknown convention %d", convention);
        return MOE_ERR_INVALID_ARG;
    }
    int64_t c = (int64_t)rows;
    if ((double)c < rows - 1e-9) c += 1;
    if (c > 0x7fffffff) {
        set_error("moe_capacity: result does not fit int32");
        return MOE_ERR_INVALID_ARG;
    }
    return (int32_t)c;
}

int moe_gate_topk(moe_handle_t *h, const void *x, const void *wg, const float *gate_bias, int32_t T,
                  float *logits_out, int32_t *topk_idx, float *topk_w, void *workspace, int64_t workspace_bytes,
                  void *stream)
{
    g_err[0] = 0;
    ProfBind bind(h);
    int rc = check_handle_T(h, T);
    if (rc != MOE_OK) return rc;
    if (T == 0) return MOE_OK;
    if (bad_ptr(x, "x") || bad_ptr(wg, "wg") || bad_ptr(gate_bias, "gate_bias", true) ||
        bad_ptr(logits_out, "logits_out", true) || bad_ptr(topk_idx, "topk_idx") || bad_ptr(topk_w, "topk_w"))
        return MOE_ERR_INVALID_ARG;
    const WsLayout L = ws_layout(h->cfg);
    float *logits_ws = nullptr;
    if (!logits_out) {
        rc = check_ws(h, workspace, workspace_bytes);
        if (rc != MOE_OK) return rc;
        logits_ws = at<float>(workspace, L.logits);
    }
    // the split-K slices of a small batch's gate GEMM live in the workspace; without one the GEMM runs whole
    float *parts = (workspace && reinterpret_cast<uintptr_t>(workspace) % 16 == 0 && workspace_bytes >= L.total)
                       ? at<float>(workspace, L.gate_parts)
                       : nullptr;
    return do_gate_topk(h, x, wg, gate_bias, T, logits_out, logits_ws, topk_idx, topk_w, (hipStream_t)stream, parts);
}

int moe_route_counts(moe_handle_t *h, const int32_t *topk_idx, int32_t T, int32_t *counts, int32_t *offsets,
                     int32_t *dst_row, int32_t *src_tok, void *workspace, int64_t workspace_bytes, void *stream)
{
    g_err[0] = 0;
    ProfBind bind(h);
    int rc = check_handle_T(h, T);
    if (rc != MOE_OK) return rc;
    const bool empty = (T == 0);  // nothing but counts and offsets is touched then
    if (bad_ptr(topk_idx, "topk_idx", empty) || bad_ptr(counts, "counts") || bad_ptr(offsets, "offsets") ||
        bad_ptr(dst_row, "dst_row", empty) || bad_ptr(src_tok, "src_tok", empty))
        return MOE_ERR_INVALID_ARG;
    rc = check_ws(h, workspace, workspace_bytes);
    if (rc != MOE_OK) return rc;
    return launch_route(topk_idx, T, h->cfg.E, h->cfg.k, counts, offsets, dst_row, src_tok,
                        at<int32_t>(workspace, ws_layout(h->cfg).block_hist), (hipStream_t)stream);
}

int moe_dispatch(moe_handle_t *h, const void *x, const int32_t *dst_row, int32_t T, void *xp, void *stream)
{
    g_err[0] = 0;
    ProfBind bind(h);
    int rc = check_handle_T(h, T);
    if (rc != MOE_OK) return rc;
    if (T == 0) return MOE_OK;
    if (bad_ptr(x, "x") || bad_ptr(dst_row, "dst_row") || bad_ptr(xp, "xp")) return MOE_ERR_INVALID_ARG;
    return launch_dispatch(h->cfg.dtype, x, dst_row, T, h->cfg.D, h->cfg.k, xp, (hipStream_t)stream);
}

int moe_expert_ffn(moe_handle_t *h, const void *xp, const int32_t *offsets, const void *w1, const void *w2,
                   const void *b1, const void *b2, int32_t n_rows, void *yp, void *workspace,
                   int64_t workspace_bytes, void *stream)
{
    g_err[0] = 0;
    ProfBind bind(h);
    if (!h) {
        set_error("handle is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    if (n_rows < 0 || (int64_t)n_rows > (int64_t)h->cfg.T_max * h->cfg.k) {
        set_error("n_rows = %d outside [0, k*T_max = %lld]", n_rows, (long long)h->cfg.T_max * h->cfg.k);
        return MOE_ERR_INVALID_ARG;
    }
    if (n_rows == 0) return MOE_OK;
    if (bad_ptr(xp, "xp") || bad_ptr(offsets, "offsets") || bad_ptr(w1, "w1") || bad_ptr(w2, "w2") ||
        bad_ptr(b1, "b1", true) || bad_ptr(b2, "b2", true) || bad_ptr(yp, "yp"))
        return MOE_ERR_INVALID_ARG;
    int rc = check_ws(h, workspace, workspace_bytes);
    if (rc != MOE_OK) return rc;
    return do_expert_ffn(h, xp, FfnExtra(), offsets, w1, w2, b1, b2, n_rows, yp, workspace, (hipStream_t)stream);
}

int moe_combine(moe_handle_t *h, const void *yp, const int32_t *dst_row, const float *topk_w, int32_t T, void *y,
                void *stream)
{
    g_err[0] = 0;
    ProfBind bind(h);
    int rc = check_handle_T(h, T);
    if (rc != MOE_OK) return rc;
    if (T == 0) return MOE_OK;
    if (bad_ptr(yp, "yp") || bad_ptr(dst_row, "dst_row") || bad_ptr(topk_w, "topk_w") || bad_ptr(y, "y"))
        return MOE_ERR_INVALID_ARG;
    return launch_combine(h->cfg.dtype, yp, dst_row, topk_w, T, h->cfg.D, h->cfg.k, y, (hipStream_t)stream);
}

static int buffered_expert_ffn(moe_handle_t *h, moe_expert_cache_t *cache, const void *xin, const int32_t *a_rows,
                               const int32_t *counts, const int32_t *offsets, const void *b1, const void *b2,
                               int32_t n_rows, void *yp, void *workspace, hipStream_t s);

// cache == NULL: experts from w1 / w2 in device memory; else buffered (w1, w2 unused)
// w1_scale != NULL: w1 / w2 are e4m3 bytes with these per-expert scales; w1_blk != NULL: e2m1 nibbles
// with these block scale bytes
static int layer_forward_impl(moe_handle_t *h, moe_expert_cache_t *cache, const void *x, const void *wg,
                              const float *gate_bias, const void *w1, const void *w2, const void *b1, const void *b2,
                              int32_t T, void *y, const moe_routing_t *routing_out, void *workspace,
                              int64_t workspace_bytes, void *stream, const float *w1_scale = nullptr,
                              const float *w2_scale = nullptr, const uint8_t *w1_blk = nullptr,
                              const uint8_t *w2_blk = nullptr)
{
    g_err[0] = 0;
    ProfBind bind(h);
    int rc = check_handle_T(h, T);
    if (rc != MOE_OK) return rc;
    const bool empty = (T == 0);  // only counts and offsets are written then
    if (bad_ptr(x, "x", empty) || bad_ptr(wg, "wg", empty) || bad_ptr(gate_bias, "gate_bias", true) ||
        bad_ptr(w1, "w1", empty || cache) || bad_ptr(w2, "w2", empty || cache) || bad_ptr(b1, "b1", true) ||
        bad_ptr(b2, "b2", true) || bad_ptr(y, "y", empty))
        return MOE_ERR_INVALID_ARG;
    moe_routing_t r;
    memset(&r, 0, sizeof(r));
    if (routing_out) r = *routing_out;
    if (bad_ptr(r.logits, "routing_out.logits", true) || bad_ptr(r.topk_idx, "routing_out.topk_idx", true) ||
        bad_ptr(r.topk_w, "routing_out.topk_w", true) || bad_ptr(r.counts, "routing_out.counts", true) ||
        bad_ptr(r.offsets, "routing_out.offsets", true) || bad_ptr(r.dst_row, "routing_out.dst_row", true) ||
        bad_ptr(r.src_tok, "routing_out.src_tok", true))
        return MOE_ERR_INVALID_ARG;
    rc = check_ws(h, workspace, workspace_bytes);
    if (rc != MOE_OK) return rc;
    const moe_config_t &c = h->cfg;
    const WsLayout L = ws_layout(c);
    hipStream_t s = (hipStream_t)stream;
    int32_t *idx = r.topk_idx ? r.topk_idx : at<int32_t>(workspace, L.topk_idx);
    float *w = r.topk_w ? r.topk_w : at<float>(workspace, L.topk_w);
    int32_t *counts = r.counts ? r.counts : at<int32_t>(workspace, L.counts);
    int32_t *offsets = r.offsets ? r.offsets : at<int32_t>(workspace, L.offsets);
    int32_t *dst_row = r.dst_row ? r.dst_row : at<int32_t>(workspace, L.dst_row);
    int32_t *src_tok = r.src_tok ? r.src_tok : at<int32_t>(workspace, L.src_tok);
    int32_t *block_hist = at<int32_t>(workspace, L.block_hist);
    void *xp = at<void>(workspace, L.xp);
    void *yp = at<void>(workspace, L.yp);

    if (empty) return launch_route(idx, 0, c.E, c.k, counts, offsets, dst_row, src_tok, block_hist, s);
    {
        // an event pair around nothing: what the bracketing itself adds to every record of this call
        ProfScope nothing("event_pair_overhead", s);
    }
    int hist_tokens = 0;  // > 0: the gate kernel has already left the expert histogram in block_hist
    rc = do_gate_topk(h, x, wg, gate_bias, T, r.logits, at<float>(workspace, L.logits), idx, w, s,
                      at<float>(workspace, L.gate_parts), block_hist, &hist_tokens);
    if (rc != MOE_OK) return rc;
    // the routing step's ranking kernel also writes the first expert GEMM's tile map (not when the
    // experts are buffered: their tile maps are per stage)
    const int64_t n_rows = (int64_t)T * c.k;
    const int wbits = cache ? cache->wbits : (w1_blk ? 4 : w1_scale ? 8 : 0);
    const int bm1 = cache ? 0
                          : gemm_variant_block_m(c.dtype, wbits ? quant_variant(wbits, n_rows, c.E)
                                                                : gemm_variant(c.dtype, n_rows, c.E, c.F, h->num_cus));
    rc = launch_route(idx, T, c.E, c.k, counts, offsets, dst_row, src_tok, block_hist, s, bm1,
                      at<int32_t>(workspace, L.tile_expert), at<int32_t>(workspace, L.tile_row),
                      at<int32_t>(workspace, L.num_tiles), bm1 > 0 ? (int)(n_rows / bm1) + c.E + 1 : 0, hist_tokens);
    if (rc != MOE_OK) return rc;
    // dispatch: a scatter of its own, or folded into the first GEMM's row addressing (then Xp is never written)
    const bool fused = fused_dispatch_ok(h, T, wbits);
    if (!fused) {
        rc = launch_dispatch(c.dtype, x, dst_row, T, c.D, c.k, xp, s);
        if (rc != MOE_OK) return rc;
    }
    if (cache) {
        rc = buffered_expert_ffn(h, cache, fused ? x : xp, fused ? src_tok : nullptr, counts, offsets, b1, b2,
                                 T * c.k, yp, workspace, s);
    } else {
        FfnExtra ex;
        ex.a_rows = fused ? src_tok : nullptr;
        ex.tile_map_ready_bm = bm1;
        ex.w1_scale = w1_scale;
        ex.w2_scale = w2_scale;
        ex.w1_blk = w1_blk;
        ex.w2_blk = w2_blk;
        rc = do_expert_ffn(h, fused ? x : xp, ex, offsets, w1, w2, b1, b2, T * c.k, yp, workspace, s);
    }
    if (rc != MOE_OK) return rc;
    return launch_combine(c.dtype, yp, dst_row, w, T, c.D, c.k, y, s);
}

int moe_layer_forward(moe_handle_t *h, const void *x, const void *wg, const float *gate_bias, const void *w1,
                      const void *w2, const void *b1, const void *b2, int32_t T, void *y,
                      const moe_routing_t *routing_out, void *workspace, int64_t workspace_bytes, void *stream)
{
    return layer_forward_impl(h, nullptr, x, wg, gate_bias, w1, w2, b1, b2, T, y, routing_out, workspace,
                              workspace_bytes, stream);
}

// moe_layer_forward for callers that cannot allocate: the workspace is the library's own scratch
// array on the handle's device.  No allocation of any kind happens here or below.
int moe_layer_forward_noalloc(moe_handle_t *h, const void *x, const void *wg, const float *gate_bias, const void *w1,
                              const void *w2, const void *b1, const void *b2, int32_t T, void *y,
                              const moe_routing_t *routing_out, void *stream)
{
    g_err[0] = 0;
    if (!h) {
        set_error("handle is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    const int64_t need = ws_layout(h->cfg).total;
    if (need > (int64_t)MOE_NOALLOC_SCRATCH_BYTES) {
        set_error("moe_layer_forward_noalloc: this handle (T_max = %d) needs %lld bytes of scratch, the library holds %lld; "
                  "use moe_layer_forward with a workspace of the caller's", h->cfg.T_max, (long long)need,
                  (long long)MOE_NOALLOC_SCRATCH_BYTES);
        return MOE_ERR_WORKSPACE;
    }
    int dev = -1;
    MOE_HIP_CHECK(hipGetDevice(&dev));
    if (dev != h->device || !h->scratch) {
        set_error("moe_layer_forward_noalloc: current device %d is not the handle's device %d", dev, h->device);
        return MOE_ERR_INVALID_ARG;
    }
    // nothing in the workspace has to start at zero: every slice is written by the call before it is read
    return layer_forward_impl(h, nullptr, x, wg, gate_bias, w1, w2, b1, b2, T, y, routing_out, h->scratch,
                              (int64_t)MOE_NOALLOC_SCRATCH_BYTES, stream);
}

// ---- 8-bit expert weights -----------------------------------------------------------------------
int moe_quantize_e4m3(moe_handle_t *h, const void *w, int32_t E, int32_t rows, int32_t cols, void *q_out,
                      float *scale_out, void *stream)
{
    g_err[0] = 0;
    if (!h) {
        set_error("handle is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    if (E < 1 || E > 65535 || rows < 16 || rows % 16 != 0 || cols < 64 || cols % 64 != 0) {
        set_error("quantize: E = %d outside [1, 65535], rows = %d not a positive multiple of 16 or cols = %d not a "
                  "positive multiple of 64", E, rows, cols);
        return MOE_ERR_INVALID_ARG;
    }
    if (bad_ptr(w, "w") || bad_ptr(q_out, "q_out") || bad_ptr(scale_out, "scale_out")) return MOE_ERR_INVALID_ARG;
    return launch_quantize_e4m3(h->cfg.dtype, w, E, rows, cols, static_cast<uint8_t *>(q_out), scale_out,
                                (hipStream_t)stream);
}

int moe_expert_ffn_w8(moe_handle_t *h, const void *xp, const int32_t *offsets, const void *w1_q, const void *w2_q,
                      const float *w1_scale, const float *w2_scale, const void *b1, const void *b2, int32_t n_rows,
                      void *yp, void *workspace, int64_t workspace_bytes, void *stream)
{
    g_err[0] = 0;
    ProfBind bind(h);
    if (!h) {
        set_error("handle is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    int rc = check_w8(h);
    if (rc != MOE_OK) return rc;
    if (n_rows < 0 || (int64_t)n_rows > (int64_t)h->cfg.T_max * h->cfg.k) {
        set_error("n_rows = %d outside [0, k*T_max = %lld]", n_rows, (long long)h->cfg.T_max * h->cfg.k);
        return MOE_ERR_INVALID_ARG;
    }
    if (n_rows == 0) return MOE_OK;
    if (bad_ptr(xp, "xp") || bad_ptr(offsets, "offsets") || bad_ptr(w1_q, "w1_q") || bad_ptr(w2_q, "w2_q") ||
        bad_ptr(w1_scale, "w1_scale") || bad_ptr(w2_scale, "w2_scale") || bad_ptr(b1, "b1", true) ||
        bad_ptr(b2, "b2", true) || bad_ptr(yp, "yp"))
        return MOE_ERR_INVALID_ARG;
    rc = check_ws(h, workspace, workspace_bytes);
    if (rc != MOE_OK) return rc;
    FfnExtra ex;
    ex.w1_scale = w1_scale;
    ex.w2_scale = w2_scale;
    return do_expert_ffn(h, xp, ex, offsets, w1_q, w2_q, b1, b2, n_rows, yp, workspace, (hipStream_t)stream);
}

int moe_layer_forward_w8(moe_handle_t *h, const void *x, const void *wg, const float *gate_bias, const void *w1_q,
                         const void *w2_q, const float *w1_scale, const float *w2_scale, const void *b1,
                         const void *b2, int32_t T, void *y, const moe_routing_t *routing_out, void *workspace,
                         int64_t workspace_bytes, void *stream)
{
    g_err[0] = 0;
    if (!h) {
        set_error("handle is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    int rc = check_w8(h);
    if (rc != MOE_OK) return rc;
    if (T > 0 && (bad_ptr(w1_scale, "w1_scale") || bad_ptr(w2_scale, "w2_scale"))) return MOE_ERR_INVALID_ARG;
    static const float one = 1.f;  // T = 0: nothing reads the scales, the pointer only selects the path
    return layer_forward_impl(h, nullptr, x, wg, gate_bias, w1_q, w2_q, b1, b2, T, y, routing_out, workspace,
                              workspace_bytes, stream, w1_scale ? w1_scale : &one, w2_scale ? w2_scale : &one);
}

// ---- 4-bit expert weights with block scales -------------------------------------------------------
int64_t moe_mxfp4_scale_bytes(int32_t rows, int32_t cols)
{
    g_err[0] = 0;
    if (rows < 32 || rows % 32 != 0 || cols < 64 || cols % 64 != 0) {
        set_error("mxfp4: rows = %d not a positive multiple of 32 or cols = %d not a positive multiple of 64", rows, cols);
        return MOE_ERR_INVALID_ARG;
    }
    return mxfp4_scale_bytes(rows, cols);
}

int moe_quantize_mxfp4(moe_handle_t *h, const void *w, int32_t E, int32_t rows, int32_t cols, void *q_out,
                       void *scale_out, void *stream)
{
    g_err[0] = 0;
    if (!h) {
        set_error("handle is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    if (E < 1 || E > 65535 || rows < 32 || rows % 32 != 0 || cols < 64 || cols % 64 != 0) {
        set_error("quantize: E = %d outside [1, 65535], rows = %d not a positive multiple of 32 or cols = %d not a "
                  "positive multiple of 64", E, rows, cols);
        return MOE_ERR_INVALID_ARG;
    }
    if (bad_ptr(w, "w") || bad_ptr(q_out, "q_out") || bad_ptr(scale_out, "scale_out")) return MOE_ERR_INVALID_ARG;
    return launch_quantize_mxfp4(h->cfg.dtype, w, E, rows, cols, static_cast<uint8_t *>(q_out),
                                 static_cast<uint8_t *>(scale_out), (hipStream_t)stream);
}

int moe_expert_ffn_w4(moe_handle_t *h, const void *xp, const int32_t *offsets, const void *w1_q, const void *w2_q,
                      const void *w1_scale, const void *w2_scale, const void *b1, const void *b2, int32_t n_rows,
                      void *yp, void *workspace, int64_t workspace_bytes, void *stream)
{
    g_err[0] = 0;
    ProfBind bind(h);
    if (!h) {
        set_error("handle is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    int rc = check_w8(h);
    if (rc != MOE_OK) return rc;
    if (n_rows < 0 || (int64_t)n_rows > (int64_t)h->cfg.T_max * h->cfg.k) {
        set_error("n_rows = %d outside [0, k*T_max = %lld]", n_rows, (long long)h->cfg.T_max * h->cfg.k);
        return MOE_ERR_INVALID_ARG;
    }
    if (n_rows == 0) return MOE_OK;
    if (bad_ptr(xp, "xp") || bad_ptr(offsets, "offsets") || bad_ptr(w1_q, "w1_q") || bad_ptr(w2_q, "w2_q") ||
        bad_ptr(w1_scale, "w1_scale") || bad_ptr(w2_scale, "w2_scale") || bad_ptr(b1, "b1", true) ||
        bad_ptr(b2, "b2", true) || bad_ptr(yp, "yp"))
        return MOE_ERR_INVALID_ARG;
    rc = check_ws(h, workspace, workspace_bytes);
    if (rc != MOE_OK) return rc;
    FfnExtra ex;
    ex.w1_blk = static_cast<const uint8_t *>(w1_scale);
    ex.w2_blk = static_cast<const uint8_t *>(w2_scale);
    return do_expert_ffn(h, xp, ex, offsets, w1_q, w2_q, b1, b2, n_rows, yp, workspace, (hipStream_t)stream);
}

int moe_layer_forward_w4(moe_handle_t *h, const void *x, const void *wg, const float *gate_bias, const void *w1_q,
                         const void *w2_q, const void *w1_scale, const void *w2_scale, const void *b1,
                         const void *b2, int32_t T, void *y, const moe_routing_t *routing_out, void *workspace,
                         int64_t workspace_bytes, void *stream)
{
    g_err[0] = 0;
    if (!h) {
        set_error("handle is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    int rc = check_w8(h);
    if (rc != MOE_OK) return rc;
    if (bad_ptr(w1_scale, "w1_scale") || bad_ptr(w2_scale, "w2_scale")) return MOE_ERR_INVALID_ARG;
    return layer_forward_impl(h, nullptr, x, wg, gate_bias, w1_q, w2_q, b1, b2, T, y, routing_out, workspace,
                              workspace_bytes, stream, nullptr, nullptr, static_cast<const uint8_t *>(w1_scale),
                              static_cast<const uint8_t *>(w2_scale));
}

// ---- expert buffering ------------------------------------------------------------------------
// bytes of one expert's W1 (= W2) as the cache stores it
static int64_t cache_half_bytes(const moe_config_t &c, int wbits)
{
    const int64_t n = (int64_t)c.F * c.D;
    return wbits == 8 ? n : wbits == 4 ? n / 2 : n * elem_size(c.dtype);
}

int64_t moe_expert_cache_bytes_q(const moe_handle_t *h, int32_t slots, int32_t wbits)
{
    g_err[0] = 0;
    if (!h || slots < 1 || (wbits != 0 && wbits != 8 && wbits != 4)) {
        set_error("handle is NULL, slots = %d < 1 or wbits = %d not 0, 8 or 4", slots, wbits);
        return MOE_ERR_INVALID_ARG;
    }
    const moe_config_t &c = h->cfg;
    return 2 * cache_index_bytes(c) + (int64_t)slots * 2 * cache_half_bytes(c, wbits);
}

int64_t moe_expert_cache_bytes(const moe_handle_t *h, int32_t slots) { return moe_expert_cache_bytes_q(h, slots, 0); }

int moe_expert_cache_create(moe_handle_t *h, int32_t slots, const void *host_w1, const void *host_w2,
                            void *device_mem, int64_t device_bytes, moe_expert_cache_t **out)
{
    return moe_expert_cache_create_q(h, slots, 0, host_w1, host_w2, nullptr, nullptr, device_mem, device_bytes, out);
}

int moe_expert_cache_create_q(moe_handle_t *h, int32_t slots, int32_t wbits, const void *host_w1, const void *host_w2,
                              const void *w1_scale, const void *w2_scale, void *device_mem, int64_t device_bytes,
                              moe_expert_cache_t **out)
{
    g_err[0] = 0;
    if (!h || !out || slots < 1 || (wbits != 0 && wbits != 8 && wbits != 4)) {
        set_error("expert cache: handle or out is NULL, slots = %d < 1 or wbits = %d not 0, 8 or 4", slots, wbits);
        return MOE_ERR_INVALID_ARG;
    }
    if (wbits != 0) {
        const int rq = check_w8(h);
        if (rq != MOE_OK) return rq;
        if (bad_ptr(w1_scale, "w1_scale") || bad_ptr(w2_scale, "w2_scale")) return MOE_ERR_INVALID_ARG;
    }
    if (bad_ptr(host_w1, "host_w1") || bad_ptr(host_w2, "host_w2") || bad_ptr(device_mem, "device_mem"))
        return MOE_ERR_INVALID_ARG;
    if (((uintptr_t)device_mem & 255) != 0 || device_bytes < moe_expert_cache_bytes_q(h, slots, wbits)) {
        set_error("expert cache: device_mem must be 256-byte aligned and hold %lld bytes (got %lld)",
                  (long long)moe_expert_cache_bytes_q(h, slots, wbits), (long long)device_bytes);
        return MOE_ERR_WORKSPACE;
    }
    const moe_config_t &c = h->cfg;
    moe_expert_cache *k = new (std::nothrow) moe_expert_cache;
    if (!k) {
        set_error("out of host memory");
        return MOE_ERR_INVALID_ARG;
    }
    k->h = h;
    k->slots = slots;
    k->host_w1 = static_cast<const uint8_t *>(host_w1);
    k->host_w2 = static_cast<const uint8_t *>(host_w2);
    k->half_bytes = cache_half_bytes(c, wbits);
    k->wbits = wbits;
    k->scale1 = w1_scale;
    k->scale2 = w2_scale;
    uint8_t *base = static_cast<uint8_t *>(device_mem);
    k->d_slot_of = reinterpret_cast<int32_t *>(base);
    k->d_stage = reinterpret_cast<int32_t *>(base + cache_index_bytes(c));
    k->d_slots = base + 2 * cache_index_bytes(c);
    k->stage_of.assign(c.E, -1);
    k->loads.assign((size_t)4 * c.E, 0);
    int rc = moe_cache_policy_create(c.E, slots, &k->policy);
    // the copy stream and the pinned block belong to the handle's device; the caller's current device is put back
    int prev_dev = -1;
    if (rc == MOE_OK && hipGetDevice(&prev_dev) != hipSuccess) rc = hip_failed(hipGetLastError(), "hipGetDevice");
    if (rc == MOE_OK && prev_dev != h->device && hipSetDevice(h->device) != hipSuccess)
        rc = hip_failed(hipGetLastError(), "hipSetDevice");
    if (rc == MOE_OK) {
        hipError_t e = hipHostMalloc(reinterpret_cast<void **>(&k->pin), (size_t)3 * c.E * 4, hipHostMallocDefault);
        if (e != hipSuccess) rc = hip_failed(e, "hipHostMalloc");
    }
    if (rc == MOE_OK) {
        hipError_t e = hipStreamCreateWithFlags(&k->copy_stream, hipStreamNonBlocking);
        if (e != hipSuccess) rc = hip_failed(e, "hipStreamCreateWithFlags");
    }
    if (prev_dev >= 0 && prev_dev != h->device) (void)hipSetDevice(prev_dev);
    if (rc != MOE_OK) {
        moe_expert_cache_destroy(k);
        return rc;
    }
    *out = k;
    return MOE_OK;
}

int moe_expert_cache_destroy(moe_expert_cache_t *k)
{
    if (!k) return MOE_OK;
    if (k->copy_stream) {
        (void)hipStreamSynchronize(k->copy_stream);
        (void)hipStreamDestroy(k->copy_stream);
    }
    for (hipEvent_t e : k->events) (void)hipEventDestroy(e);
    if (k->pin) (void)hipHostFree(k->pin);
    if (k->policy) moe_cache_policy_destroy(k->policy);
    delete k;
    return MOE_OK;
}

int moe_expert_cache_reset(moe_expert_cache_t *k)
{
    g_err[0] = 0;
    if (!k) {
        set_error("expert cache is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    k->bytes_copied = k->stages = 0;
    return moe_cache_policy_reset(k->policy);
}

int moe_expert_cache_stats(const moe_expert_cache_t *k, int64_t *hits, int64_t *misses, int64_t *bytes_copied,
                           int64_t *stages)
{
    g_err[0] = 0;
    if (!k) {
        set_error("expert cache is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    if (bytes_copied) *bytes_copied = k->bytes_copied;
    if (stages) *stages = k->stages;
    return moe_cache_policy_stats(k->policy, hits, misses, nullptr);
}

// The expert FFN from the cache's slots.  Host-side order of work:
//   counts -> host (one wait for the stream), cache decision, index arrays -> device, then per
//   policy stage: the stage's missing experts are copied on the copy stream (after everything that
//   ran in earlier stages, whose slots they may take), the stage's resident experts compute
//   meanwhile on the caller's stream, and the copied ones follow once their copy has landed.
static int buffered_expert_ffn_run(moe_handle_t *h, moe_expert_cache_t *k, const void *xin, const int32_t *a_rows,
                                   const int32_t *counts, const int32_t *offsets, const void *b1, const void *b2,
                                   int32_t n_rows, void *yp, void *workspace, hipStream_t s, bool *policy_advanced);

static int buffered_expert_ffn(moe_handle_t *h, moe_expert_cache_t *k, const void *xin, const int32_t *a_rows,
                               const int32_t *counts, const int32_t *offsets, const void *b1, const void *b2,
                               int32_t n_rows, void *yp, void *workspace, hipStream_t s)
{
    bool policy_advanced = false;
    const int rc = buffered_expert_ffn_run(h, k, xin, a_rows, counts, offsets, b1, b2, n_rows, yp, workspace, s,
                                           &policy_advanced);
    if (rc != MOE_OK && policy_advanced) {
        // The cache decision already counts the missed experts as resident, but a copy or a launch after it
        // failed: forget every resident expert, so that the next call loads what it needs instead of running
        // on slots whose contents never arrived.  (Copies already enqueued finish before the slots are reused:
        // the next call waits for the caller's stream and orders its copies behind the copy stream's work.)
        (void)hipStreamSynchronize(k->copy_stream);
        (void)moe_cache_policy_reset(k->policy);
    }
    return rc;
}

static int buffered_expert_ffn_run(moe_handle_t *h, moe_expert_cache_t *k, const void *xin, const int32_t *a_rows,
                                   const int32_t *counts, const int32_t *offsets, const void *b1, const void *b2,
                                   int32_t n_rows, void *yp, void *workspace, hipStream_t s, bool *policy_advanced)
{
    const moe_config_t &c = h->cfg;
    if (k->h != h) {
        set_error("the expert cache belongs to another handle");
        return MOE_ERR_INVALID_ARG;
    }
    const int E = c.E;
    int32_t *h_counts = k->pin, *h_slot = k->pin + E, *h_launch = k->pin + 2 * E;
    MOE_HIP_CHECK(hipMemcpyAsync(h_counts, counts, (size_t)E * 4, hipMemcpyDeviceToHost, s));
    MOE_HIP_CHECK(hipStreamSynchronize(s));  // also: every earlier call's reads of the slots are over
    int32_t n_loads = 0, n_stages = 0;
    int rc = cache_policy_step(k->policy, h_counts, h_slot, k->stage_of.data(), k->loads.data(), E, &n_loads, &n_stages);
    *policy_advanced = true;
    if (rc != MOE_OK) return rc;
    // launch index of an expert: 2 * stage for residents, 2 * stage + 1 for the ones copied in this batch
    std::vector<int> in_launch((size_t)2 * (n_stages > 0 ? n_stages : 1), 0);
    for (int e = 0; e < E; ++e) h_launch[e] = k->stage_of[e] < 0 ? -1 : 2 * k->stage_of[e];
    for (int i = 0; i < n_loads; ++i) h_launch[k->loads[4 * i]] += 1;
    for (int e = 0; e < E; ++e)
        if (h_launch[e] >= 0) in_launch[h_launch[e]] += 1;
    MOE_HIP_CHECK(hipMemcpyAsync(k->d_slot_of, h_slot, (size_t)E * 4, hipMemcpyHostToDevice, s));
    MOE_HIP_CHECK(hipMemcpyAsync(k->d_stage, h_launch, (size_t)E * 4, hipMemcpyHostToDevice, s));

    FfnExtra ex;
    ex.a_rows = a_rows;
    ex.b_slot = k->d_slot_of;
    ex.stage_of = k->d_stage;
    // stride between slots in the GEMM's unit for B: elements for elem weights, bytes for 8 and 4 bits
    ex.slot_stride = k->wbits ? 2 * k->half_bytes : 2 * (int64_t)c.F * c.D;
    if (k->wbits == 8) {
        ex.w1_scale = static_cast<const float *>(k->scale1);
        ex.w2_scale = static_cast<const float *>(k->scale2);
    } else if (k->wbits == 4) {
        ex.w1_blk = static_cast<const uint8_t *>(k->scale1);
        ex.w2_blk = static_cast<const uint8_t *>(k->scale2);
    }
    const void *w1 = k->d_slots, *w2 = k->d_slots + k->half_bytes;
    hipEvent_t last_done = nullptr;
    size_t ev = 0;
    int li = 0;  // next entry of the load list (it is ordered by stage)
    for (int st = 0; st < n_stages; ++st) {
        hipEvent_t loaded = nullptr;
        if (li < n_loads && k->loads[4 * li + 3] == st) {
            if (last_done) MOE_HIP_CHECK(hipStreamWaitEvent(k->copy_stream, last_done, 0));
            for (; li < n_loads && k->loads[4 * li + 3] == st; ++li) {
                const int e = k->loads[4 * li], slot = k->loads[4 * li + 1];
                uint8_t *dst = k->d_slots + (int64_t)slot * 2 * k->half_bytes;
                MOE_HIP_CHECK(hipMemcpyAsync(dst, k->host_w1 + (int64_t)e * k->half_bytes, (size_t)k->half_bytes,
                                             hipMemcpyHostToDevice, k->copy_stream));
                MOE_HIP_CHECK(hipMemcpyAsync(dst + k->half_bytes, k->host_w2 + (int64_t)e * k->half_bytes,
                                             (size_t)k->half_bytes, hipMemcpyHostToDevice, k->copy_stream));
                k->bytes_copied += 2 * k->half_bytes;
            }
            rc = cache_event(k, ev++, &loaded);
            if (rc != MOE_OK) return rc;
            MOE_HIP_CHECK(hipEventRecord(loaded, k->copy_stream));
        }
        for (int part = 0; part < 2; ++part) {
            if (in_launch[2 * st + part] == 0) continue;
            if (part == 1) MOE_HIP_CHECK(hipStreamWaitEvent(s, loaded, 0));
            ex.stage = 2 * st + part;
            rc = do_expert_ffn(h, xin, ex, offsets, w1, w2, b1, b2, n_rows, yp, workspace, s);
            if (rc != MOE_OK) return rc;
            rc = cache_event(k, ev++, &last_done);
            if (rc != MOE_OK) return rc;
            MOE_HIP_CHECK(hipEventRecord(last_done, s));
        }
        k->stages += 1;
    }
    return MOE_OK;
}

int moe_layer_forward_buffered(moe_handle_t *h, moe_expert_cache_t *cache, const void *x, const void *wg,
                               const float *gate_bias, const void *b1, const void *b2, int32_t T, void *y,
                               const moe_routing_t *routing_out, void *workspace, int64_t workspace_bytes,
                               void *stream)
{
    if (!cache) {
        g_err[0] = 0;
        set_error("expert cache is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    return layer_forward_impl(h, cache, x, wg, gate_bias, nullptr, nullptr, b1, b2, T, y, routing_out, workspace,
                              workspace_bytes, stream);
}

int64_t moe_static_workspace_bytes(const moe_handle_t *h, int32_t T, int32_t capacity, int32_t mode)
{
    g_err[0] = 0;
    if (!h) {
        set_error("handle is NULL");
        return MOE_ERR_INVALID_ARG;
    }
    if (T < 0 || T > h->cfg.T_max || capacity < 1 || (int64_t)capacity * h->cfg.E > 0x3fffffff) {
        set_error("T = %d or capacity = %d out of range", T, capacity);
        return MOE_ERR_INVALID_ARG;
    }
    if (mode != MOE_STATIC_EINSUM && mode != MOE_STATIC_INDEXED) {
        set_error("unknown static mode %d", mode);
        return MOE_ERR_INVALID_ARG;
    }
    return static_layout(h->cfg, T, capacity, mode).total;
}

int moe_layer_forward_static(moe_handle_t *h, const void *x, const void *wg, const float *gate_bias, const void *w1,
                             const void *w2, const void *b1, const void *b2, int32_t T, int32_t capacity, int32_t mode,
                             void *y, int32_t *dropped_count, const moe_routing_t *routing_out, void *workspace,
                             int64_t workspace_bytes, void *stream)
{
    g_err[0] = 0;
    ProfBind bind(h);
    int rc = check_handle_T(h, T);
    if (rc != MOE_OK) return rc;
    const moe_config_t &c = h->cfg;
    if (capacity < 1 || (int64_t)capacity * c.E > 0x3fffffff) {
        set_error("capacity = %d out of range", capacity);
        return MOE_ERR_INVALID_ARG;
    }
    if (mode != MOE_STATIC_EINSUM && mode != MOE_STATIC_INDEXED) {
        set_error("unknown static mode %d", mode);
        return MOE_ERR_INVALID_ARG;
    }
    hipStream_t s = (hipStream_t)stream;
    if (bad_ptr(dropped_count, "dropped_count", true)) return MOE_ERR_INVALID_ARG;
    if (T == 0) return dropped_count ? launch_fill_u32(dropped_count, 1, 0, s) : MOE_OK;
    if (bad_ptr(x, "x") || bad_ptr(wg, "wg") || bad_ptr(gate_bias, "gate_bias", true) || bad_ptr(w1, "w1") ||
        bad_ptr(w2, "w2") || bad_ptr(b1, "b1", true) || bad_ptr(b2, "b2", true) || bad_ptr(y, "y"))
        return MOE_ERR_INVALID_ARG;
    moe_routing_t r;
    memset(&r, 0, sizeof(r));
    if (routing_out) r = *routing_out;
    if (bad_ptr(r.logits, "routing_out.logits", true) || bad_ptr(r.topk_idx, "routing_out.topk_idx", true) ||
        bad_ptr(r.topk_w, "routing_out.topk_w", true) || bad_ptr(r.counts, "routing_out.counts", true) ||
        bad_ptr(r.offsets, "routing_out.offsets", true) || bad_ptr(r.dst_row, "routing_out.dst_row", true))
        return MOE_ERR_INVALID_ARG;
    const StaticLayout L = static_layout(c, T, capacity, mode);
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 != 0) {
        set_error("workspace is NULL or not 256-byte aligned");
        return MOE_ERR_WORKSPACE;
    }
    if (workspace_bytes < L.total) {
        set_error("workspace has %lld bytes, %lld needed", (long long)workspace_bytes, (long long)L.total);
        return MOE_ERR_WORKSPACE;
    }
    void *ws = workspace;
    const int64_t R = (int64_t)c.E * capacity;
    int32_t *idx = r.topk_idx ? r.topk_idx : at<int32_t>(ws, L.topk_idx);
    float *w = r.topk_w ? r.topk_w : at<float>(ws, L.topk_w);
    int32_t *counts_s = r.counts ? r.counts : at<int32_t>(ws, L.counts_s);
    int32_t *offsets_s = r.offsets ? r.offsets : at<int32_t>(ws, L.offsets_s);
    int32_t *slot_row = r.dst_row ? r.dst_row : at<int32_t>(ws, L.slot_row);
    int32_t *dropped = dropped_count ? dropped_count : at<int32_t>(ws, L.num_tiles) + 1;  // spare word of the slot
    int32_t *idx_t = at<int32_t>(ws, L.idx_t);
    int32_t *pos = at<int32_t>(ws, L.pos);
    int32_t *offsets_static = at<int32_t>(ws, L.offsets_static);
    void *xd = at<void>(ws, L.xd);
    void *yd = at<void>(ws, L.yd);

    rc = do_gate_topk(h, x, wg, gate_bias, T, r.logits, at<float>(ws, L.logits), idx, w, s);
    if (rc != MOE_OK) return rc;
    // slot of every assignment = its rank inside its expert in slot-major order
    rc = launch_transpose_idx(idx, T, c.k, idx_t, dropped, s);
    if (rc != MOE_OK) return rc;
    rc = launch_route(idx_t, T * c.k, c.E, 1, counts_s, offsets_s, pos, at<int32_t>(ws, L.src_s),
                      at<int32_t>(ws, L.block_hist), s);
    if (rc != MOE_OK) return rc;
    rc = launch_static_rows(idx_t, pos, offsets_s, T, c.k, c.E, capacity, slot_row, dropped, s);
    if (rc != MOE_OK) return rc;
    rc = launch_static_offsets(offsets_static, c.E, capacity, s);
    if (rc != MOE_OK) return rc;

    GemmParams p;
    if (mode == MOE_STATIC_INDEXED) {
        int32_t *row_tok = at<int32_t>(ws, L.row_tok);
        rc = launch_fill_u32(row_tok, R, 0xffffffffu, s);
        if (rc != MOE_OK) return rc;
        rc = launch_row_tokens(slot_row, T, c.k, row_tok, s);
        if (rc != MOE_OK) return rc;
        rc = launch_padded_gather(c.dtype, x, row_tok, R, c.D, xd, s);
        if (rc != MOE_OK) return rc;
    } else {
        // dispatch = one-hot mask [E*cap, T] times x: Xd[r,:] = sum_t mask[r,t] * x[t,:]
        const int64_t es = elem_size(c.dtype);
        void *mask = at<void>(ws, L.mask);
        void *cw = at<void>(ws, L.cw);
        void *xt = at<void>(ws, L.xt);
        rc = launch_fill_u32(mask, R * L.ldt * es / 4, 0, s);
        if (rc != MOE_OK) return rc;
        rc = launch_fill_u32(cw, (int64_t)T * L.ldk * es / 4, 0, s);
        if (rc != MOE_OK) return rc;
        rc = launch_static_masks(c.dtype, slot_row, w, T, c.k, mask, L.ldt, cw, L.ldk, s);
        if (rc != MOE_OK) return rc;
        rc = launch_transpose_pad(c.dtype, x, T, c.D, xt, L.ldt, s);
        if (rc != MOE_OK) return rc;
        memset(&p, 0, sizeof(p));
        p.name = "static_dispatch_einsum";
        p.A = mask;
        p.lda = L.ldt;
        p.B = xt;
        p.ldb = L.ldt;
        p.C = xd;
        p.ldc = c.D;
        p.M = (int)R;
        p.N = c.D;
        p.K = (int)L.ldt;
        rc = launch_gemm(c.dtype, p, false, 0, c.dtype == MOE_DTYPE_F32, false, h->num_cus, s);
        if (rc != MOE_OK) return rc;
    }
    // every expert processes all of its `capacity` rows, zero rows included
    rc = run_expert_ffn(h, xd, FfnExtra(), offsets_static, w1, w2, b1, b2, R, yd, at<void>(ws, L.hd),
                        at<int32_t>(ws, L.tile_expert), at<int32_t>(ws, L.tile_row), at<int32_t>(ws, L.num_tiles), s);
    if (rc != MOE_OK) return rc;
    if (mode == MOE_STATIC_INDEXED) return launch_combine(c.dtype, yd, slot_row, w, T, c.D, c.k, y, s);
    // combine = weight mask [T, E*cap] times the expert outputs
    void *ydt = at<void>(ws, L.ydt);
    rc = launch_transpose_pad(c.dtype, yd, R, c.D, ydt, L.ldk, s);
    if (rc != MOE_OK) return rc;
    memset(&p, 0, sizeof(p));
    p.name = "static_combine_einsum";
    p.A = at<void>(ws, L.cw);
    p.lda = L.ldk;
    p.B = ydt;
    p.ldb = L.ldk;
    p.C = y;
    p.ldc = c.D;
    p.M = T;
    p.N = c.D;
    p.K = (int)L.ldk;
    return launch_gemm(c.dtype, p, false, 0, c.dtype == MOE_DTYPE_F32, false, h->num_cus, s);
}

}  // extern "C"
