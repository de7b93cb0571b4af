/*
 * moe.h -- C ABI of the dynamically gated Mixture-of-Experts layer forward for
 * AMD MI355X (gfx950), one GPU.
 *
 * The layer follows "Towards MoE Deployment: Mitigating Inefficiencies in
 * Mixture-of-Expert (MoE) Inference": a linear gate picks the top-k experts of
 * every token (Sec. 2.3, Sec. 2.4); with DYNAMIC gating (Sec. 5.1) the expert
 * assignments are sorted by expert, the occurrences of each expert are counted,
 * the tokens are reordered by the sort index into variable-sized per-expert
 * batches (no capacity, no dropped token, no placeholder row), the experts run
 * on exactly their rows, and the original order is restored by indexing.  The
 * STATIC gating the paper replaces (Sec. 3.2, Sec. 5.1: fixed capacity per
 * expert, one-hot dispatch masks multiplied with the tokens, drops and zero
 * padding) is exported as a baseline for comparison.  Expert Buffering (Sec. 6:
 * expert parameters in host memory behind a small device cache) is at the end.
 *
 * Conventions for every call
 *   - Plain C.  Returns MOE_OK (0) or a negative MOE_ERR_* code; after an error
 *     moe_last_error() gives a message (thread-local, valid until the next call
 *     on the thread).  No exception crosses this boundary.
 *   - Every tensor argument is a DEVICE pointer owned by the caller, row-major,
 *     densely packed, 16-byte aligned.  The library allocates no device memory in
 *     any call below; scratch comes from the caller's `workspace` (device memory,
 *     256-byte aligned, at least moe_workspace_bytes() long; contents undefined
 *     before and after a call; one workspace must not be used by two calls that
 *     may overlap in time).
 *   - Calls only enqueue work on `stream` (a hipStream_t passed as void*; NULL =
 *     the default stream) and never wait for the device or read device data on
 *     the host -- except moe_profile_end and moe_layer_forward_buffered, which say
 *     so.  Argument errors are found on the host before anything is launched.
 *   - "elem" below is the storage type named by moe_config_t.dtype: float for
 *     MOE_DTYPE_F32, bfloat16 bit patterns for MOE_DTYPE_BF16.  Accumulation is
 *     always fp32; gate logits and gate weights are always fp32.
 *   - Notation: T tokens, D = token (model) dimension, F = expert hidden
 *     dimension, E experts, k experts per token, N = k*T assignments.
 *   - Inputs must be finite.  Expert indices handed to moe_route_counts must lie
 *     in [0,E); values outside are clamped into the range (memory safe, result
 *     then meaningless).  The k experts of one token must be distinct, as top-k
 *     selection makes them (Sec. 2.3); a token that names an expert twice still
 *     gets two rows of that expert, in slot order, for any batch size.
 */
#ifndef MOE355_MOE_H
#define MOE355_MOE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_OK 0
#define MOE_ERR_INVALID_ARG (-1) /* NULL / misaligned pointer, T outside [0,T_max], bad size */
#define MOE_ERR_UNSUPPORTED (-2) /* dtype, k, E, D or F outside the supported set */
#define MOE_ERR_WORKSPACE (-3)   /* workspace missing or too small */
#define MOE_ERR_HIP (-4)         /* the HIP runtime reported a failure */

#define MOE_DTYPE_F32 0
#define MOE_DTYPE_BF16 1

#define MOE_STATIC_EINSUM 0  /* one-hot dispatch / combine masks multiplied as dense GEMMs */
#define MOE_STATIC_INDEXED 1 /* same capacity, padding and drops, rows moved by index */

#define MOE_CAPACITY_PAPER 0 /* capacity = ceil(cf * T): the paper's C*S */
#define MOE_CAPACITY_SHARE 1 /* capacity = ceil(cf * k*T / E): cf times an expert's fair share */

#define MOE_MAX_K 8
#define MOE_MAX_E 1024

/* Shape of the layer.  Supported: dtype in {F32, BF16}; 1 <= E <= MOE_MAX_E;
 * 1 <= k <= min(E, MOE_MAX_K); D and F positive multiples of 8; T_max >= 0 with
 * k*T_max < 2^30 (row indices are int32). */
typedef struct moe_config {
    int32_t T_max;       /* largest T any call on this handle will be given */
    int32_t D;
    int32_t F;
    int32_t E;
    int32_t k;
    int32_t dtype;       /* MOE_DTYPE_* */
    int32_t renormalize; /* 1: gate weights = softmax over the k selected logits (sum to 1);
                            0: the k selected entries of the softmax over all E logits */
} moe_config_t;

typedef struct moe_handle moe_handle_t; /* opaque: the config plus device properties */

/* Optional routing outputs of the fused calls; every member may be NULL. */
typedef struct moe_routing {
    float *logits;     /* [T,E]  */
    int32_t *topk_idx; /* [T,k]  */
    float *topk_w;     /* [T,k]  */
    int32_t *counts;   /* [E]    */
    int32_t *offsets;  /* [E+1]  */
    int32_t *dst_row;  /* [T,k]  */
    int32_t *src_tok;  /* [k*T]  */
} moe_routing_t;

/* Create / destroy a handle (host memory only).  moe_create validates the config
 * (MOE_ERR_UNSUPPORTED / MOE_ERR_INVALID_ARG) and queries the current device
 * (MOE_ERR_HIP when there is none). */
int moe_create(const moe_config_t *cfg, moe_handle_t **out);
int moe_destroy(moe_handle_t *h);

/* Message of the last error on this thread ("" if none). */
const char *moe_last_error(void);

/* Per-kernel timing for benchmarks (Sec. 3.1 of the paper reports a latency breakdown by
 * component; this is the tool that produces one here).  Between moe_profile_begin and
 * moe_profile_end every kernel the calls on this handle launch is bracketed by HIP events
 * recorded on the call's stream (at most 64 records; later launches are not recorded).
 * moe_profile_end is the one call of this library that WAITS for the device: it waits for the
 * recorded events, writes the elapsed milliseconds of record i to ms_out[i] (i < max_records),
 * stores the number of records in *n_records and switches profiling off.  moe_profile_name
 * gives the kernel name of record i ("" when out of range); valid until the next begin.  The fused
 * layer calls start with one record named "event_pair_overhead" that brackets no kernel at all: the
 * time an event pair itself adds to each of the other records. */
int moe_profile_begin(moe_handle_t *h);
int moe_profile_end(moe_handle_t *h, float *ms_out, int32_t max_records, int32_t *n_records);
const char *moe_profile_name(const moe_handle_t *h, int32_t i);

/* Bytes of workspace that make every dynamic-gating call on this handle succeed for
 * any T <= T_max (routing scratch, the dispatched rows Xp [N,D], the hidden rows
 * H [N,F] and the expert outputs Yp [N,D]).  Negative error code on a bad handle. */
int64_t moe_workspace_bytes(const moe_handle_t *h);

/* Same for moe_layer_forward_static with the given T, capacity and mode. */
int64_t moe_static_workspace_bytes(const moe_handle_t *h, int32_t T, int32_t capacity, int32_t mode);

/* Rows per expert for a capacity factor cf under one of the two conventions
 * (MOE_CAPACITY_PAPER: Sec. 3 / Sec. 5.1, capacity = C*S, e.g. S = 6, C = 0.5 -> 3;
 * MOE_CAPACITY_SHARE: cf * k*T/E).  Negative error code on bad arguments. */
int32_t moe_capacity(int32_t T, int32_t E, int32_t k, double cf, int32_t convention);

/* Gate + top-k routing decision (Sec. 2.3, Sec. 2.4).
 *   logits[t,e] = sum_d x[t,d] * wg[e,d] (+ gate_bias[e]),  fp32
 *   topk_idx[t,0..k-1] = the k experts with the largest logit, slot 0 the largest,
 *                        equal logits to the lower expert index
 *   topk_w[t,j] = gate weight of slot j (see moe_config_t.renormalize), fp32
 * x [T,D] elem, wg [E,D] elem, gate_bias [E] fp32 or NULL.  logits_out [T,E] fp32 may
 * be NULL only if `workspace` is given (kernels that need the logits in memory keep them
 * there; for bf16, E <= 128, D a multiple of 64 and more than 256 tokens the decision is
 * taken in the gate GEMM's epilogue and the logits are written only where logits_out asks
 * for them).  workspace may be NULL when logits_out is given.  T = 0 is a no-op. */
int moe_gate_topk(moe_handle_t *h, const void *x, const void *wg, const float *gate_bias,
                  int32_t T, float *logits_out, int32_t *topk_idx, float *topk_w,
                  void *workspace, int64_t workspace_bytes, void *stream);

/* Routing metadata of dynamic gating (Sec. 5.1: the sort index of the expert
 * assignments and the number of occurrences of each expert).
 *   counts[e]    = number of (t,j) with topk_idx[t,j] = e                (sums to k*T)
 *   offsets[e]   = counts[0] + ... + counts[e-1],  offsets[E] = k*T
 *   dst_row[t,j] = offsets[e] + number of tokens t' < t that selected e,  e = topk_idx[t,j]
 *   src_tok[r]   = the token whose assignment landed in row r (inverse of dst_row)
 * The permutation is the stable one (ascending token inside each expert) and is
 * computed without atomics on global memory, so it is identical from run to run.
 * All arrays int32.  Needs the workspace.  T = 0 writes zero counts and offsets. */
int moe_route_counts(moe_handle_t *h, const int32_t *topk_idx, int32_t T,
                     int32_t *counts, int32_t *offsets, int32_t *dst_row, int32_t *src_tok,
                     void *workspace, int64_t workspace_bytes, void *stream);

/* Dispatch (Sec. 5.1: reorder the inputs by the sort index; they are then split by the
 * counts, i.e. rows [offsets[e], offsets[e+1]) of xp are expert e's batch):
 *   xp[dst_row[t,j], :] = x[t, :]      x [T,D] elem -> xp [k*T, D] elem.
 * Every row of xp is written exactly once; nothing is padded or dropped. */
int moe_dispatch(moe_handle_t *h, const void *x, const int32_t *dst_row, int32_t T,
                 void *xp, void *stream);

/* Grouped expert FFN on the dispatched rows (Sec. 2.2 FFN block; each expert processes
 * only the tokens assigned to it, Sec. 5.1):
 *   for r in [offsets[e], offsets[e+1]):  yp[r,:] = W2[e] * relu(W1[e] * xp[r,:] + b1[e]) + b2[e]
 * xp [N,D], w1 [E,F,D], w2 [E,D,F], b1 [E,F] or NULL, b2 [E,D] or NULL, yp [N,D], all elem;
 * offsets [E+1] int32 on the device with offsets[E] = N = k*T, N given by the caller as
 * n_rows (it sizes the launch; the device never reads more than offsets says).
 * Experts with an empty range are skipped and their weights are never read.
 * The hidden rows are rounded to elem once after the ReLU.  Needs the workspace. */
int moe_expert_ffn(moe_handle_t *h, const void *xp, const int32_t *offsets,
                   const void *w1, const void *w2, const void *b1, const void *b2,
                   int32_t n_rows, void *yp, void *workspace, int64_t workspace_bytes, void *stream);

/* Combine (Sec. 5.1: restore the original order by indexing, weighted by the gate):
 *   y[t,:] = sum_{j=0..k-1, in this order} topk_w[t,j] * yp[dst_row[t,j], :]
 * accumulated in fp32 and rounded once.  yp [k*T,D] elem -> y [T,D] elem. */
int moe_combine(moe_handle_t *h, const void *yp, const int32_t *dst_row, const float *topk_w,
                int32_t T, void *y, void *stream);

/* The whole dynamically gated layer: gate_topk -> route_counts -> dispatch ->
 * expert_ffn -> combine, enqueued back to back on `stream` with no host
 * synchronisation.  y [T,D] elem.  routing_out (may be NULL) receives the routing
 * arrays whose members are non-NULL. */
int moe_layer_forward(moe_handle_t *h, const void *x, const void *wg, const float *gate_bias,
                      const void *w1, const void *w2, const void *b1, const void *b2,
                      int32_t T, void *y, const moe_routing_t *routing_out,
                      void *workspace, int64_t workspace_bytes, void *stream);

/* moe_layer_forward for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops (one decode step after the other), harnesses that
 * forbid hipMalloc.  Same arguments minus the workspace, same kernels, same result bit for bit.  The
 * scratch is an array of MOE_NOALLOC_SCRATCH_BYTES bytes that lives inside the library, once per GPU
 * the library runs on, until the process ends; the call allocates nothing (no hipMalloc / hipFree,
 * no allocating library routine) and still only enqueues work on `stream`.
 *   - The handle's moe_workspace_bytes() must fit: MOE_ERR_WORKSPACE otherwise (a handle made for
 *     decode-sized batches does: T_max = 64, D = 2048, F = 8192, E = 128, k = 2 needs 3.6 MB).
 *   - The current device must be the one the handle was created on (MOE_ERR_INVALID_ARG otherwise).
 *   - Every such call on one GPU uses the same array: calls that may overlap in time on one GPU
 *     (different streams, different threads, different handles) race.  The array keeps the previous
 *     call's contents; nothing in it has to be cleared between calls. */
#define MOE_NOALLOC_SCRATCH_BYTES (8 * 1024 * 1024)
int moe_layer_forward_noalloc(moe_handle_t *h, const void *x, const void *wg, const float *gate_bias,
                              const void *w1, const void *w2, const void *b1, const void *b2,
                              int32_t T, void *y, const moe_routing_t *routing_out, void *stream);

/* Static-capacity baseline (Sec. 3.2, Sec. 5.1): same gate; every expert owns
 * `capacity` rows; assignments are placed slot by slot (all first choices in token
 * order, then all second choices, ...) into the first empty row of their expert and
 * are DROPPED when the expert is full (they then contribute nothing; gate weights are
 * not renormalised); unused rows are zero and the experts still process all
 * E*capacity rows.
 *   MOE_STATIC_EINSUM : dispatch = one-hot mask [E*cap, T] times x, combine = weight
 *                       mask [T, E*cap] times the expert outputs, both as dense GEMMs
 *                       (the formulation the paper identifies as the inefficiency);
 *   MOE_STATIC_INDEXED: same rows, moved by index.
 * dropped_count (device int32, may be NULL) receives the number of dropped assignments.
 * routing_out (may be NULL): logits, topk_idx, topk_w as in the dynamic call; counts[e] = assignments
 * of expert e BEFORE dropping, offsets = their exclusive scan; dst_row[t,j] = e*capacity + row inside
 * the expert, or -1 for a dropped assignment; src_tok is not written.
 * EINSUM mode needs masks of (E*capacity) x T and T x (E*capacity) elements in the workspace.
 * Workspace: moe_static_workspace_bytes(). */
int moe_layer_forward_static(moe_handle_t *h, const void *x, const void *wg, const float *gate_bias,
                             const void *w1, const void *w2, const void *b1, const void *b2,
                             int32_t T, int32_t capacity, int32_t mode, void *y,
                             int32_t *dropped_count, const moe_routing_t *routing_out,
                             void *workspace, int64_t workspace_bytes, void *stream);

/* ---- Weight-only 8-bit expert weights (an extension for the weight-streaming regime; not in ----
 * ---- the paper: its decoder steps, Sec. 4, are bound by reading expert parameters)          ---- */

/* W[e] ~ scale[e] * q[e]: q are OCP e4m3 bytes (1 sign, 4 exponent, 3 mantissa bits, no infinity,
 * largest value 448), scale[e] is the smallest power of two with max|W[e]| / scale[e] <= 448 (1 for
 * an all-zero expert), q = W / scale rounded to nearest even.
 * w [E, rows, cols] elem (device), scale_out [E] fp32 (device), q_out E * rows * cols bytes (device)
 * in a blocked layout made for the grouped GEMM's loads: inside expert e, the byte of element
 * (n, k) sits at  ((n / 16) * (cols / 64) + k / 64) * 1024 + (n % 16) * 64 + k % 64,  i.e. 16 rows
 * x 64 columns form one contiguous 1 KB block and the blocks of a 16-row group follow each other
 * along the columns.  rows a multiple of 16, cols a multiple of 64 (MOE_ERR_INVALID_ARG otherwise).
 * Enqueued on `stream`. */
int moe_quantize_e4m3(moe_handle_t *h, const void *w, int32_t E, int32_t rows, int32_t cols, void *q_out,
                      float *scale_out, void *stream);

/* moe_expert_ffn / moe_layer_forward with such weights: w1_q (from W1 [E,F,D]: rows = F, cols = D)
 * and w2_q (from W2 [E,D,F]: rows = D, cols = F) in the layout above, w1_scale, w2_scale [E] fp32.  Activations, biases and outputs stay elem = bf16; every e4m3 value is a bf16
 * value, so the products are those of the dequantised weights, accumulated in fp32 and multiplied
 * by the scale once per output.  Needs dtype bf16 and D, F multiples of 64 (MOE_ERR_UNSUPPORTED
 * otherwise).  Halves the parameter bytes a step reads; meant for small batches per expert. */
int moe_expert_ffn_w8(moe_handle_t *h, const void *xp, const int32_t *offsets, const void *w1_q, const void *w2_q,
                      const float *w1_scale, const float *w2_scale, const void *b1, const void *b2, int32_t n_rows,
                      void *yp, void *workspace, int64_t workspace_bytes, void *stream);
int moe_layer_forward_w8(moe_handle_t *h, const void *x, const void *wg, const float *gate_bias, const void *w1_q,
                         const void *w2_q, const float *w1_scale, const float *w2_scale, const void *b1,
                         const void *b2, int32_t T, void *y, const moe_routing_t *routing_out, void *workspace,
                         int64_t workspace_bytes, void *stream);

/* ---- Weight-only 4-bit expert weights with block scales (the OCP microscaling layout; an ----
 * ---- extension like the 8-bit one above, not in the paper)                               ---- */

/* Every 32 consecutive elements of a weight row share one scale: W[n][32 b + i] ~ s[n][b] * v[n][32 b + i].
 * v are e2m1 codes (4 bits: bit 3 sign, bits 2..0 -> 0, 0.5, 1, 1.5, 2, 3, 4, 6); s[n][b] is the
 * smallest power of two with max|block| <= 6 s (nothing saturates), stored as the byte e with
 * s = 2^(e - 127), e >= 1, e = 127 for an all-zero block; v = W / s rounded to nearest, ties to the
 * even code.
 * w [E, rows, cols] elem (device).  q_out: E * rows * cols / 2 bytes (device); inside expert e the
 * element (n, k) is nibble (k % 2) (low nibble first) of byte
 *   ((n / 32) * (cols / 64) + k / 64) * 1024 + (n % 32) * 32 + (k % 64) / 2,
 * i.e. 32 rows x 64 columns form one contiguous 1 KB block and the blocks of a 32-row group follow
 * each other along the columns.  scale_out: E * moe_mxfp4_scale_bytes(rows, cols) bytes (device);
 * inside expert e the scale of (n, block b) is byte
 *   ((n / 32) * ceil(cols / 512) + b / 16) * 512 + (n % 32) * 16 + b % 16
 * (bytes of blocks past the last column are padding and unspecified).
 * rows a multiple of 32, cols a multiple of 64 (MOE_ERR_INVALID_ARG otherwise).  Enqueued on `stream`. */
int64_t moe_mxfp4_scale_bytes(int32_t rows, int32_t cols);
int moe_quantize_mxfp4(moe_handle_t *h, const void *w, int32_t E, int32_t rows, int32_t cols, void *q_out,
                       void *scale_out, void *stream);

/* moe_expert_ffn / moe_layer_forward with such weights (w1_q, w1_scale from W1 [E,F,D]: rows = F,
 * cols = D; w2_q, w2_scale from W2 [E,D,F]: rows = D, cols = F).  s * v is exactly a bf16 number, so
 * the products are those of the dequantised weights, accumulated in fp32.  Activations, biases and
 * outputs stay bf16.  Needs dtype bf16 and D, F multiples of 64 (MOE_ERR_UNSUPPORTED otherwise).
 * A quarter of the parameter bytes of bf16 weights per step. */
int moe_expert_ffn_w4(moe_handle_t *h, const void *xp, const int32_t *offsets, const void *w1_q, const void *w2_q,
                      const void *w1_scale, const void *w2_scale, const void *b1, const void *b2, int32_t n_rows,
                      void *yp, void *workspace, int64_t workspace_bytes, void *stream);
int moe_layer_forward_w4(moe_handle_t *h, const void *x, const void *wg, const float *gate_bias, const void *w1_q,
                         const void *w2_q, const void *w1_scale, const void *w2_scale, const void *b1,
                         const void *b2, int32_t T, void *y, const moe_routing_t *routing_out, void *workspace,
                         int64_t workspace_bytes, void *stream);

/* ---- Expert Buffering (Sec. 6): expert parameters in host memory, a device cache of a few ----
 * ---- experts, copies overlapped with expert computation                                   ---- */

/* Cache management alone (host logic, no device work; Sec. 6 "Cache Management").  The experts
 * with counts[e] > 0 are active and are visited in increasing id order: a resident expert is a
 * hit; a miss goes to a free slot, else it replaces a victim -- residents that are not active in
 * this batch first, then active ones, inside each class the one that entered the cache last
 * (Last In, First Out; with 2 slots and experts (1,2,3) needed, 3 replaces 2 and 1 stays).
 *   counts   [E] host int32
 *   slot_of  [E] host int32 out: slot the expert runs from in this batch, -1 if not active
 *   stage_of [E] host int32 out: execution stage, -1 if not active.  A victim that already ran
 *            in this batch must finish before its slot is overwritten, so its replacement is one
 *            stage later; stages never decrease along the id order; experts of one stage have
 *            distinct slots
 *   loads    [4*max_loads] host int32 out: (expert, slot, victim or -1, stage) per miss, in order
 * Errors: MOE_ERR_INVALID_ARG for NULL arguments or a load list that is too short (n_loads then
 * holds the needed length; the cache state has still advanced).  The object is owned by the
 * caller and not thread safe. */
typedef struct moe_cache_policy moe_cache_policy_t;
int moe_cache_policy_create(int32_t E, int32_t slots, moe_cache_policy_t **out);
int moe_cache_policy_destroy(moe_cache_policy_t *p);
int moe_cache_policy_reset(moe_cache_policy_t *p); /* empty cache, zero statistics */
int moe_cache_policy_step(moe_cache_policy_t *p, const int32_t *counts, int32_t *slot_of, int32_t *stage_of,
                          int32_t *loads, int32_t max_loads, int32_t *n_loads, int32_t *n_stages);
/* hits / misses since creation or reset (an access = one active expert of one batch);
 * slot_expert [slots] host int32 (may be NULL) receives the expert held by every slot, -1 = free. */
int moe_cache_policy_stats(const moe_cache_policy_t *p, int64_t *hits, int64_t *misses, int32_t *slot_expert);

/* The device side of the buffer.  host_w1 [E,F,D] and host_w2 [E,D,F] (elem) stay in HOST memory
 * owned by the caller -- pinned memory (hipHostMalloc), or the copies are not asynchronous -- and
 * must stay valid and unchanged while the cache lives.  device_mem is device memory owned by the
 * caller, at least moe_expert_cache_bytes(h, slots) bytes, 256-byte aligned: `slots` slots of one
 * expert's W1 and W2 plus two small index arrays.  The object creates one copy stream (default
 * priority) and a few events; destroy it before the handle. */
typedef struct moe_expert_cache moe_expert_cache_t;
int64_t moe_expert_cache_bytes(const moe_handle_t *h, int32_t slots);
int moe_expert_cache_create(moe_handle_t *h, int32_t slots, const void *host_w1, const void *host_w2,
                            void *device_mem, int64_t device_bytes, moe_expert_cache_t **out);
/* The same buffer over quantised expert weights (the 8- and 4-bit formats further up; not in the
 * paper, which buffers the parameters as they are): the host link carries half / a quarter of the
 * bytes per missed expert.  wbits = 8: host_w1 / host_w2 are the e4m3 bytes of moe_quantize_e4m3
 * (E * F * D each), w1_scale / w2_scale its fp32 scales [E]; wbits = 4: the e2m1 bytes of
 * moe_quantize_mxfp4 (E * F * D / 2 each) and its block scale bytes.  The scales of ALL experts stay
 * in DEVICE memory (w1_scale, w2_scale: device pointers, valid while the cache lives; they are at
 * most 1/16 of the data); only the data bytes are buffered.  wbits = 0: as moe_expert_cache_create
 * (scales NULL).  Needs what the quantised calls need (MOE_ERR_UNSUPPORTED otherwise).
 * moe_layer_forward_buffered then runs the quantised expert GEMMs. */
int64_t moe_expert_cache_bytes_q(const moe_handle_t *h, int32_t slots, int32_t wbits);
int moe_expert_cache_create_q(moe_handle_t *h, int32_t slots, int32_t wbits, const void *host_w1, const void *host_w2,
                              const void *w1_scale, const void *w2_scale, void *device_mem, int64_t device_bytes,
                              moe_expert_cache_t **out);
int moe_expert_cache_destroy(moe_expert_cache_t *c);
int moe_expert_cache_reset(moe_expert_cache_t *c); /* forget every resident expert, zero the statistics */
/* hits, misses, bytes copied host to device, and stages executed, since creation or reset */
int moe_expert_cache_stats(const moe_expert_cache_t *c, int64_t *hits, int64_t *misses, int64_t *bytes_copied,
                           int64_t *stages);

/* moe_layer_forward with buffered experts (Sec. 6): same result, bit for bit, as the plain call
 * on the same parameters.  After the routing step the per-expert token counts are copied to the
 * host and the call WAITS for `stream` once (the cache decision is host logic, as in the paper,
 * where the counts reach the host with the first all-to-all); missing experts are then copied into
 * their slots on the cache's copy stream while the experts that are already resident compute, and
 * the expert FFN runs stage by stage (see moe_cache_policy_step) from the slots.  b1 [E,F] and
 * b2 [E,D] (NULL or device memory) are not buffered.  Needs `slots` >= 1; a batch with more active
 * experts than slots runs in several stages.  Calls on one cache must not overlap.  If the call fails after
 * the cache decision was taken (a copy or a launch reports an error), the cache forgets every resident expert
 * (hit / miss statistics are zeroed with it), so the next call reloads what it needs. */
int moe_layer_forward_buffered(moe_handle_t *h, moe_expert_cache_t *cache, const void *x, const void *wg,
                               const float *gate_bias, const void *b1, const void *b2, int32_t T, void *y,
                               const moe_routing_t *routing_out, void *workspace, int64_t workspace_bytes,
                               void *stream);

/* ---- Load-balancing placement (Sec. 7): which device hosts which expert ---- */

/* Host logic on historical activation data; no device work.  A [E,B] host fp32, row-major:
 * A[m*B + b] = fraction of batch b's tokens that went to expert m.  Every device gets E / n_devices
 * experts (E must divide evenly).  Experts are taken in descending order of their average load
 * (equal: lower id first) and put on the device that offers the smallest load (equal: lower device
 * id); a full device leaves the candidates.
 *   greedy (Sec. 7.1):          the load of a device is the sum of its experts' average loads;
 *   anticorrelation (Sec. 7.2): for the current expert a, the load of a device is the sum over its
 *                               experts m of average[m] + corr_weight * S[a][m], S the Pearson
 *                               correlation of the two experts' activations (0 for an expert that
 *                               never varies); the paper uses corr_weight = 0.5.
 * device_of [E] host int32 out.  MOE_ERR_INVALID_ARG on NULL pointers or sizes that do not fit. */
int moe_placement_greedy(const float *A, int32_t E, int32_t B, int32_t n_devices, int32_t *device_of);
int moe_placement_anticorrelation(const float *A, int32_t E, int32_t B, int32_t n_devices, double corr_weight,
                                  int32_t *device_of);
/* Max Load = the largest share of a batch that any device receives, over all batches; Avg Max
 * Load = the largest share per batch, averaged over the batches (Sec. 7.1).  Outputs may be NULL. */
int moe_placement_loads(const float *A, int32_t E, int32_t B, const int32_t *device_of, int32_t n_devices,
                        double *max_load, double *avg_max_load);

#ifdef __cplusplus
}
#endif
#endif /* MOE355_MOE_H */
