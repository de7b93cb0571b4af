// bf16 MFMA GEMM  C = A * B^T (+ bias, ReLU)  with fp32 accumulation, plain or grouped.
//
// Serves the three dense contractions of the layer: the gate (x * Wg^T, fp32 logits out), and the
// two grouped expert GEMMs (Xp * W1[e]^T with ReLU, H * W2[e]^T), where every expert multiplies
// exactly the rows dynamic gating gave it (paper Sec. 5.1) -- no capacity padding.
//
// Both operands are K-contiguous, so every MFMA operand fragment (8 consecutive bf16 along K for
// one row) is one 16-byte LDS read.  Tile: BM x BN x 64, WM x WN waves of 64 lanes, each wave owns
// a (BM/WM) x (BN/WN) sub-tile made of 32x32 MFMA blocks (v_mfma_f32_32x32x16_bf16).  The weight
// fragment is the MFMA's first operand and the activation fragment the second, so a lane ends up
// with 4 CONSECUTIVE output columns of one output row per group of 4 accumulator registers and
// stores them as one 8-byte (bf16) or 16-byte (fp32) access.
//
// LDS layout: tile rows of 64 bf16 = 128 B = 8 chunks of 16 B; chunk c of row r is stored at
// chunk position c ^ ((r >> 1) & 7).  gfx950's LDS serves a 16-byte-per-lane read 16 consecutive
// lanes (256 B, 64 banks) per clock: the 16 rows such a group reads at one K chunk are 8 even rows
// (first half of the banks) and 8 odd rows (second half), and the swizzle gives each half 8
// different chunk positions, so fragment reads are conflict free (measured: 4 clk per
// ds_read_b128 against 6 clk with an (r & 7) swizzle).
//
// Three K pipelines, chosen per tile shape (template argument STAGES):
//  * ring of K steps (the 256x256 tiles of the grouped GEMM, STAGES = DTL16): v_mfma_f32_16x16x32_bf16
//    instead of the 32x32 blocks, operands straight into LDS, five slots of one 32-wide K step, one
//    load every seventh MFMA (four per step); described where it is implemented, inside the kernel.
//  * direct-to-LDS, whole K tiles (small tiles, the gate): STAGES LDS stages; K tiles go straight from global
//    memory into LDS (global_load_lds_dwordx4, no register staging), the loads run STAGES-1 K
//    tiles ahead of the MFMAs and are waited for (vmcnt) only at the barrier that ends an
//    iteration.  Several such blocks share a CU, so one block's load burst and barrier hide
//    behind another block's MFMAs.
//  * register-staged (256- and 128-row tiles, one or two blocks per CU): measured on gfx950, a
//    vector-memory instruction costs the issuing wave 20-30 clocks of MFMA issue and the CU's
//    address unit 16 clocks, so a K tile's loads issued as one burst stall every wave while the
//    matrix units idle, and with only two 64 KB stages in LDS they cannot be issued late either.
//    Here the loads of K tile i+2 go into registers one by one between the MFMAs of iteration i,
//    are written to the other LDS buffer at the same slot of iteration i+1 and the register is
//    refilled at once: every load has a full iteration to land and the address unit sees an
//    even stream.
// In the last two, the fragments of K-step ks+1 are read while the MFMAs of K-step ks issue (the
// instruction order is pinned with sched_group_barrier / sched_barrier, otherwise the compiler
// sinks the reads next to their use).
//
// Epilogue (bf16 output, last two pipelines): each wave converts a 32-row strip of its tile, parks it in the LDS rows
// only this wave's loads ever fill, and writes it out with 16 bytes per lane, i.e. whole
// contiguous row segments per store instruction; the scattered form (16 bytes per row per
// instruction) cost up to a fifth of a tile's time.
//
// Launch: PERSISTENT.  The grid is (CUs x resident blocks per CU); workgroups are handed to the 8
// XCDs round-robin and each XCD has its own L2, so XCD x walks the contiguous range
// [x*chunk, (x+1)*chunk) of the logical tile list, its blocks taking consecutive entries.  The
// list orders tiles GROUP_M M-tiles at a time across all N-tiles, so the tiles an XCD works on
// together share A rows and B (weight) rows.  The load cursor walks the block's whole sequence of (tile, K tile)
// pairs, so the first K tiles of the NEXT tile are loaded during the last iterations of the current
// one: the pipeline never drains between tiles and the epilogue's stores overlap the next tile.
#include <mutex>

#include "moe_internal.h"

namespace moe355 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
// Types for reading operand fragments out of LDS.  The compiler orders an LDS read that carries type-based
// alias information after EVERY direct-to-LDS load in flight (s_waitcnt vmcnt(0) in front of the read), which
// drains the load pipeline once per K tile; reads through vector types and may_alias types carry none, and
// the explicit vmcnt before each stage barrier is what orders them.
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef uint32_t __attribute__((may_alias)) u32_lds;
typedef uint16_t __attribute__((may_alias)) u16_lds;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) void glb_void;

// One 32-bit word at an address that is the same for every lane of the wave, through the scalar data path
// (read only).  The compiler issues such loads as vector loads here (it cannot prove that the kernel's own
// stores leave the tile map alone), and a vector load's result can only be waited for together with every
// vector load issued before it -- at a tile switch that drains the whole operand pipeline.  The scalar path
// has its own counter.  The words read were written by an earlier kernel.
__device__ __forceinline__ int32_t uniform_load(const int32_t *ptr)
{
    int32_t v;
    asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(ptr) : "memory");
    return v;
}
// two independent words with one wait
__device__ __forceinline__ void uniform_load2(const int32_t *pa, const int32_t *pb, int32_t &a, int32_t &b)
{
    asm volatile("s_load_dword %0, %2, 0x0\n\ts_load_dword %1, %3, 0x0\n\ts_waitcnt lgkmcnt(0)"
                 : "=&s"(a), "=&s"(b)
                 : "s"(pa), "s"(pb)
                 : "memory");
}

static constexpr int BK = 64;
static constexpr int GROUP_M = 4;
static constexpr int REG_STAGED = 0;  // value of the STAGES template argument that selects the register-staged pipeline
static constexpr int DTL16 = -1;      // ... and the one that selects 16x16x32 MFMAs out of a ring of K-step slots filled by direct-to-LDS loads
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ uint32_t to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ float from_bf16(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
// two fp32 -> packed bf16, round to nearest even (one v_cvt_pk_bf16_f32)
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    const bf16x2 b = __builtin_convertvector(v, bf16x2);
    return *reinterpret_cast<const uint32_t *>(&b);
}

// max(x, 0) on two packed bf16: a bf16 is negative exactly when its bit pattern is negative as a 16-bit integer,
// so one packed integer max replaces two fp32 compares (and the canonicalisation the compiler puts in front of
// them); rounding is monotonic and keeps zero, so ReLU after the conversion equals ReLU before it.
typedef __attribute__((ext_vector_type(2))) short i16x2;
__device__ __forceinline__ uint32_t relu_bf16x2(uint32_t packed)
{
    const i16x2 zero = {0, 0};
    const i16x2 r = __builtin_elementwise_max(*reinterpret_cast<const i16x2 *>(&packed), zero);
    return *reinterpret_cast<const uint32_t *>(&r);
}

struct TileInfo {
    int row0, row_end, expert, n0;
    int kt0, split;  // plain mode with split K: first K tile and index of this block's K range
};

// BQ: storage of the B operand (the weights).  0: bf16.  8: 8-bit floats (OCP e4m3, one byte per
// element, a tile row of 64 elements = 64 bytes) with one fp32 scale per expert; a fragment is
// widened to bf16 in registers after the LDS read (every e4m3 value is a bf16 value, so the products
// are exact) and the scale multiplies the fp32 accumulators in the epilogue.  4: 4-bit floats (OCP
// e2m1, two per byte, a tile row = 32 bytes) with one power-of-two scale byte (e8m0) per 32
// elements along K; the scale is applied while widening (v_cvt_scalef32_pk_bf16_fp4), the result is
// again exactly a bf16 value.  8 and 4: direct-to-LDS pipeline only.
template <int BM, int BN, int WM, int WN, bool OUT_F32, bool RELU, bool GROUPED, bool KFULL, int MINB, int STAGES,
          int BQ = 0>
__global__ __launch_bounds__(WM *WN * 64, MINB) void gemm_bf16_kernel(GemmParams p)
{
    constexpr int THREADS = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int MI = WTM / 32, NI = WTN / 32;
    constexpr bool B8 = BQ == 8, B4 = BQ == 4;
    static_assert(BQ == 0 || B8 || B4, "B storage: bf16, e4m3 or e2m1");
    constexpr int A_IT = BM * 8 / THREADS, B_IT = (B8 ? BN * 4 : B4 ? BN * 2 : BN * 8) / THREADS;
    constexpr int BROW = B8 ? BK / 2 : B4 ? BK / 4 : BK;  // one B tile row in 16-bit units
    constexpr int BTILE = BN * BROW;                       // one B stage in 16-bit units
    static_assert(!B8 || (BN * 4) % THREADS == 0, "8-bit B tile rows must split evenly over threads");
    static_assert(!B4 || (BN * 2) % THREADS == 0, "4-bit B tile rows must split evenly over threads");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be made of 32x32 blocks");
    static_assert((BM * 8) % THREADS == 0 && (BN * 8) % THREADS == 0, "tile rows must split evenly over threads");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem_raw[];
    // STAGES == REG_STAGED selects the register-staged pipeline (two LDS buffers)
    constexpr bool RSTAGE = STAGES == REG_STAGED;
    constexpr bool D16 = STAGES == DTL16;
    constexpr int NSTAGE = (RSTAGE || D16) ? 2 : STAGES;
    uint16_t *sA = reinterpret_cast<uint16_t *>(smem_raw);  // [NSTAGE][BM*64]
    uint16_t *sB = sA + NSTAGE * BM * BK;                   // [NSTAGE][BN*64]
    static_assert(NSTAGE >= 2, "at least two LDS stages");
    static_assert(!RSTAGE || KFULL, "the register-staged pipeline needs K to be a multiple of the K tile");
    static_assert(!D16 || (KFULL && BQ == 0 && !OUT_F32), "the 16x16x32 pipeline: bf16 in and out, K a multiple of the K tile");
    static_assert(BQ == 0 || (KFULL && !RSTAGE && GROUPED), "8- and 4-bit weights: grouped direct-to-LDS pipeline, K a multiple of the K tile");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int K = p.K;
    // Split K (plain mode, skinny problems: the gate GEMM of a decoder step has a tile or two and a long K
    // loop): the K tiles are cut into k_split equal ranges, each a tile of its own whose fp32 result goes to
    // its own slice (range 0 to C, range i > 0 to c_parts + (i - 1) * split_stride); whoever reads C adds the
    // slices in order.
    const int S = (!GROUPED && p.k_split > 1) ? p.k_split : 1;
    const int KT = (K + BK - 1) / BK / S;  // the launcher made sure that S divides the K tile count

    // ---- the block's sequence of tiles -----------------------------------------------------------
    // Tail splitting (grouped GEMM over 256x256 tiles): a persistent launch of G blocks runs
    // ceil(tiles / G) rounds, and when the last round is mostly empty the chip idles for a whole
    // tile time.  So the launch with tail_mode 1 stops at the last whole round, and a second launch
    // (tail_mode 2, a smaller tile shape, more blocks per CU) runs the L leftover tiles as SUB
    // sub-tiles each.  Both compute the same cut from the device-side tile count; the split is taken
    // when the sub-tiles' lower rate still beats one more whole round (measured: a tail of L tiles
    // costs 1.5 to 1.7 x L / G rounds, so it is taken for L < G / 1.8).
    constexpr int PT = 256;                             // parent tile edge
    constexpr int SUB_N = PT / BN > 0 ? PT / BN : 1;    // sub-tiles per parent along N
    constexpr int SUB = (PT / BM > 0 ? PT / BM : 1) * SUB_N;
    const bool tail_sub = GROUPED && p.tail_mode == 2;
    const int n_tiles = (p.N + (tail_sub ? PT : BN) - 1) / (tail_sub ? PT : BN);  // of the tile list's geometry
    const int m_tiles = GROUPED ? p.num_tiles[0] : (p.M + BM - 1) / BM;
    int live = m_tiles * n_tiles * S;          // logical tiles
    int cut = 0;                               // first parent tile of the tail
    if (GROUPED && (p.tail_mode == 1 || p.tail_mode == 2)) {
        const int left = live % p.main_slots;
        cut = (left > 0 && left * 9 < p.main_slots * 5) ? live - left : live;
        live = tail_sub ? (live - cut) * SUB : cut;
    }
    const int chunk = (live + 7) >> 3;         // per XCD
    const int xcd = blockIdx.x & 7;
    const int slots = gridDim.x >> 3;          // blocks per XCD (grid is a multiple of 8)
    int seq = blockIdx.x >> 3;                 // position inside the XCD's chunk
    auto seq_ok = [&](int sq) { return sq < chunk && xcd * chunk + sq < live; };
    // logical tile -> (M tile, N tile): groups of GROUP_M M-tiles (the last group may be narrower),
    // inside a group the M index runs fastest
    auto tile_info = [&](int sq) {
        int lid = xcd * chunk + sq;
        int sub = 0, split = 0;
        if (S > 1) {
            split = lid % S;
            lid /= S;
        }
        if (tail_sub) {
            sub = lid % SUB;
            lid = cut + lid / SUB;
        }
        const int per_group = GROUP_M * n_tiles;
        const int grp = lid / per_group;
        const int within = lid - grp * per_group;
        const int gsz = min(GROUP_M, m_tiles - grp * GROUP_M);
        const int mt = grp * GROUP_M + within % gsz;
        const int nt = within / gsz;
        TileInfo t;
        if (GROUPED) {
            uniform_load2(p.tile_expert + mt, p.tile_row + mt, t.expert, t.row0);
            t.row_end = uniform_load(p.offsets + t.expert + 1);
        } else {
            t.expert = 0;
            t.row0 = mt * BM;
            t.row_end = p.M;
        }
        t.n0 = nt * BN;
        t.kt0 = split * KT;
        t.split = split;
        if (tail_sub) {  // sub-tile (sub / SUB_N, sub % SUB_N) of the 256x256 parent
            t.row0 += (sub / SUB_N) * BM;
            t.n0 = nt * PT + (sub % SUB_N) * BN;
        }
        return t;
    };
    if (GROUPED && !OUT_F32 && p.c_zero_row >= 0 && blockIdx.x == 0 && p.tail_mode != 2) {
        // one all-zero row behind the output rows, for the GEMM that reads C as its A (N is a multiple of 8)
        uint16_t *z = static_cast<uint16_t *>(p.C) + (int64_t)p.c_zero_row * p.ldc;
        for (int i = tid * 8; i < p.N; i += THREADS * 8) *reinterpret_cast<uint4 *>(z + i) = make_uint4(0, 0, 0, 0);
    }
    if (!seq_ok(seq)) return;

    const uint16_t *Ag = static_cast<const uint16_t *>(p.A);
    const uint16_t *Bg0 = static_cast<const uint16_t *>(p.B);

    f32x16 acc[MI][NI];
    auto zero_acc = [&]() {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
    };

    // fragment read offsets: row = (wave tile) + mi*32 + (lane & 31), K chunk = ks*2 + (lane >> 5)
    const int frag_row = lane & 31;
    const int frag_half = lane >> 5;
    const int swz = (lane >> 1) & 7;  // == (row >> 1) & 7 for every row this lane reads

    // MFMAs of one K tile out of LDS stage `cur`.
    // 4-bit weights: the block scales are staged in LDS too, behind the operand stages: two buffers of
    // 16 bytes per weight row of the tile (the scales of 8 consecutive K tiles, two 32-element blocks per K
    // tile), one for the 8 K tiles being computed (c_buf) and one being filled for the 8 after them.
    // (Kept in registers instead, the refill every 8th K tile made the compiler wait for the load it had
    // just issued -- a full memory latency with the whole operand pipeline drained.)
    uint8_t *sS = reinterpret_cast<uint8_t *>(sB + NSTAGE * BTILE);
    static_assert(!B4 || BN * 16 == (THREADS / 64) * 1024, "one 1 KB scale load per wave covers the tile's rows");
    int c_buf = 0;
    auto compute = [&](int cur, int kt) {
        const uint16_t *cA = sA + cur * BM * BK + (wm * WTM + frag_row) * BK;
        const uint16_t *cB = sB + cur * BTILE + (wn * WTN + frag_row) * BROW;
        (void)kt;
        uint32_t sc2[B4 ? NI : 1];
        if constexpr (B4) {
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                sc2[ni] = *reinterpret_cast<const u16_lds *>(sS + c_buf * (BN * 16) + (wn * WTN + ni * 32 + frag_row) * 16 +
                                                             ((kt & 7) << 1));
        }
        (void)sc2;
        bf16x8 af[2][MI], bfr[2][NI];
        auto load_frags = [&](int ks, int set) {
            const int chunkpos = ((ks * 2 + frag_half) ^ swz) << 3;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                af[set][mi] = *reinterpret_cast<const bf16x8 *>(cA + mi * 32 * BK + chunkpos);
            if constexpr (B8) {
                // 64-byte rows, 16-byte chunk c of row r at chunk position c ^ ((r >> 2) & 3); the 8
                // bytes of this lane's fragment: chunk ks, half frag_half
                const int bytepos = ((ks ^ ((lane >> 2) & 3)) << 4) + (frag_half << 3);
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    const u32x2 raw = *reinterpret_cast<const u32x2 *>(reinterpret_cast<const uint8_t *>(cB) +
                                                                       ni * 32 * (BK) + bytepos);
                    const f32x2 f0 = __builtin_amdgcn_cvt_pk_f32_fp8(raw.x, false);
                    const f32x2 f1 = __builtin_amdgcn_cvt_pk_f32_fp8(raw.x, true);
                    const f32x2 f2 = __builtin_amdgcn_cvt_pk_f32_fp8(raw.y, false);
                    const f32x2 f3 = __builtin_amdgcn_cvt_pk_f32_fp8(raw.y, true);
                    const uint4 packed = make_uint4(pack_bf16(f0[0], f0[1]), pack_bf16(f1[0], f1[1]),
                                                    pack_bf16(f2[0], f2[1]), pack_bf16(f3[0], f3[1]));
                    bfr[set][ni] = *reinterpret_cast<const bf16x8 *>(&packed);
                }
            } else if constexpr (B4) {
                // 32-byte rows; this lane's 8 elements of K-step ks are the 4 bytes at ks*8 + half*4, their
                // block scale is byte (kt mod 8)*2 + ks/2 of the row's 16 scale bytes (sc2: the K tile's two)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    const uint32_t raw = *reinterpret_cast<const u32_lds *>(reinterpret_cast<const uint8_t *>(cB) +
                                                                            ni * 32 * (BK / 2) + ks * 8 + frag_half * 4);
                    const float scale = __uint_as_float(((sc2[ni] >> ((ks >> 1) << 3)) & 0xffu) << 23);  // 2^(byte - 127)
                    const bf16x2 d0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(raw, scale, 0);
                    const bf16x2 d1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(raw, scale, 1);
                    const bf16x2 d2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(raw, scale, 2);
                    const bf16x2 d3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(raw, scale, 3);
                    const uint4 packed = make_uint4(*reinterpret_cast<const uint32_t *>(&d0),
                                                    *reinterpret_cast<const uint32_t *>(&d1),
                                                    *reinterpret_cast<const uint32_t *>(&d2),
                                                    *reinterpret_cast<const uint32_t *>(&d3));
                    bfr[set][ni] = *reinterpret_cast<const bf16x8 *>(&packed);
                }
            } else {
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    bfr[set][ni] = *reinterpret_cast<const bf16x8 *>(cB + ni * 32 * BK + chunkpos);
            }
        };
        load_frags(0, 0);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            if (ks + 1 < BK / 16) load_frags(ks + 1, (ks + 1) & 1);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ks & 1][ni], af[ks & 1][mi], acc[mi][ni],
                                                                          0, 0, 0);
            // issue order: one LDS read behind each of the first MFMAs, then the remaining MFMAs
            if (ks + 1 < BK / 16) {
                constexpr int NR = MI + NI, NM = MI * NI;
#pragma unroll
                for (int i = 0; i < (NR < NM ? NR : NM); ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                }
                if (NR > NM) __builtin_amdgcn_sched_group_barrier(0x100, NR - NM, 0);
                if (NM > NR) __builtin_amdgcn_sched_group_barrier(0x008, NM - NR, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- epilogue: acc[mi][ni] holds D[column][row]: lane -> row (lane & 31) of block mi, registers
    // 4g..4g+3 -> columns 8g + 4*(lane >> 5) + 0..3 of block ni
    // A wave tile of 256 accumulator registers lives in the accumulation registers (AGPRs); left to
    // itself the compiler copies all of them to VGPRs at the loop exit and spills.  Reading them one
    // by one where they are used keeps the epilogue at a handful of VGPRs.  The reads are opaque to
    // the compiler's hazard handling, so the MFMA -> accumulator-read distance is padded by hand.
    constexpr bool ACC_IN_AGPR = MI * NI * 16 > 128;
    auto epilogue = [&](const TileInfo &t) {
        if constexpr (ACC_IN_AGPR) {
            asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
        }
        const uint16_t *bias = static_cast<const uint16_t *>(p.bias);
        if (bias) bias += (int64_t)t.expert * p.strideBias;
        const float b_scale = (B8 && p.b_scale) ? __int_as_float(uniform_load(reinterpret_cast<const int32_t *>(p.b_scale) + t.expert)) : 1.f;
        (void)b_scale;
        const bool vec_ok = !OUT_F32 || ((p.ldc & 3) == 0 && (p.N & 3) == 0);
        // The fp32 offsets of this lane's columns are fetched before the first store: a load
        // issued between stores would have to wait for every store before it (memory operations
        // of a wave complete in order), once per group of four columns.
        float bias32[NI][4][4];
        const bool add_bias32 = p.bias_f32 && t.split == 0;
        if (add_bias32) {
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int col = t.n0 + wn * WTN + ni * 32 + 8 * g + 4 * (lane >> 5);
#pragma unroll
                    for (int i = 0; i < 4; ++i) bias32[ni][g][i] = (col + i < p.N) ? p.bias_f32[col + i] : 0.f;
                }
            // Added here, under the same condition as the loads and for every row block, not inside the
            // row / column predicates below: a loaded register whose use sits behind a branch that a wave may
            // skip counts as "load still in flight" for the rest of the kernel, and the compiler then waits
            // for ALL loads (vmcnt(0)) before it reuses that register -- at the top of every K iteration.
            if constexpr (!ACC_IN_AGPR) {
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[mi][ni][r] += bias32[ni][r >> 2][r & 3];
            }
        }
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int row = t.row0 + wm * WTM + mi * 32 + (lane & 31);
            if (row >= t.row_end) continue;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int col = t.n0 + wn * WTN + ni * 32 + 8 * g + 4 * (lane >> 5);
                    if (col >= p.N) continue;
                    float v[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if constexpr (ACC_IN_AGPR)
                            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v[i]) : "a"(acc[mi][ni][4 * g + i]));
                        else
                            v[i] = acc[mi][ni][4 * g + i];
                    }
                    if constexpr (B8) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[i] *= b_scale;
                    }
                    if (bias) {
                        if (col + 3 < p.N) {
                            const uint2 bb = *reinterpret_cast<const uint2 *>(bias + col);
                            v[0] += __uint_as_float(bb.x << 16);
                            v[1] += __uint_as_float(bb.x & 0xffff0000u);
                            v[2] += __uint_as_float(bb.y << 16);
                            v[3] += __uint_as_float(bb.y & 0xffff0000u);
                        } else {
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                if (col + i < p.N) v[i] += from_bf16(bias[col + i]);
                        }
                    }
                    if constexpr (ACC_IN_AGPR) {
                        if (add_bias32) {
#pragma unroll
                            for (int i = 0; i < 4; ++i) v[i] += bias32[ni][g][i];
                        }
                    }
                    if (RELU && OUT_F32) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[i] = v[i] > 0.f ? v[i] : 0.f;
                    }
                    if (OUT_F32) {
                        float *c = (t.split == 0 ? static_cast<float *>(p.C) : p.c_parts + (int64_t)(t.split - 1) * p.split_stride) +
                                   (int64_t)row * p.ldc + col;
                        if (vec_ok) {
                            *reinterpret_cast<float4 *>(c) = make_float4(v[0], v[1], v[2], v[3]);
                        } else {
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                if (col + i < p.N) c[i] = v[i];
                        }
                    } else {
                        // bf16 output: N and ldc are multiples of 8 here, so the 4 columns exist
                        uint2 o;
                        o.x = pack_bf16(v[0], v[1]);
                        o.y = pack_bf16(v[2], v[3]);
                        if (RELU) {
                            o.x = relu_bf16x2(o.x);
                            o.y = relu_bf16x2(o.y);
                        }
                        *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(p.C) + (int64_t)row * p.ldc + col) = o;
                    }
                }
            }
        }
    };

    // ---- bf16 epilogue through LDS: a wave turns one 32-row strip of its tile (32 x WTN outputs)
    // into bf16, parks it in LDS and stores it back out with 16 bytes per lane, so a store
    // instruction writes whole contiguous row segments instead of 32 scattered 16-byte pieces.
    // The strip lives in the rows of the just-consumed LDS stage that THIS wave's own loads fill
    // (rows (wave*IT + i)*8..+7), so no other wave ever writes there and no barrier is needed: the
    // wave's own LDS accesses execute in order, all waves finished reading that stage before the
    // last barrier, and the wave's next load into it is issued after the strip's last read returned.
    // 16-byte chunk c of strip row r sits at chunk position c ^ (r mod chunks-per-row).
    constexpr int STRIP_ROW_BYTES = WTN * 2;
    constexpr int STRIP_BYTES = 32 * STRIP_ROW_BYTES;
    constexpr bool STRIP_IN_A = A_IT * 1024 >= STRIP_BYTES;
    constexpr bool STRIP_IN_B = !STRIP_IN_A && B_IT * 1024 >= STRIP_BYTES;
    constexpr bool LDS_EPILOGUE = !OUT_F32 && KFULL && (STRIP_IN_A || STRIP_IN_B);
    auto epilogue_lds = [&](const TileInfo &t, int free_stage) {
        constexpr int CPRW = STRIP_ROW_BYTES / 16;  // chunks per strip row
        constexpr int RPI = 64 / CPRW;              // strip rows one 64-lane access covers
        if constexpr (ACC_IN_AGPR) asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
        uint8_t *stg = reinterpret_cast<uint8_t *>(STRIP_IN_A ? sA + free_stage * BM * BK + wave * A_IT * 8 * BK
                                                             : sB + free_stage * BTILE + wave * B_IT * 8 * BK);
        const uint16_t *bias = static_cast<const uint16_t *>(p.bias);
        if (bias) bias += (int64_t)t.expert * p.strideBias;
        const float b_scale = (B8 && p.b_scale) ? __int_as_float(uniform_load(reinterpret_cast<const int32_t *>(p.b_scale) + t.expert)) : 1.f;
        (void)b_scale;
        const int r = lane & 31;
        const int col_base = t.n0 + wn * WTN;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int cl = ni * 32 + 8 * g + 4 * (lane >> 5);  // column inside the strip
                    const int col = col_base + cl;
                    float v[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if constexpr (ACC_IN_AGPR)
                            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v[i]) : "a"(acc[mi][ni][4 * g + i]));
                        else
                            v[i] = acc[mi][ni][4 * g + i];
                    }
                    if constexpr (B8) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[i] *= b_scale;
                    }
                    if (bias && col < p.N) {  // N is a multiple of 8 for bf16 output: the 4 columns exist together
                        const uint2 bb = *reinterpret_cast<const uint2 *>(bias + col);
                        v[0] += __uint_as_float(bb.x << 16);
                        v[1] += __uint_as_float(bb.x & 0xffff0000u);
                        v[2] += __uint_as_float(bb.y << 16);
                        v[3] += __uint_as_float(bb.y & 0xffff0000u);
                    }
                    if (p.bias_f32 && col < p.N) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[i] += p.bias_f32[col + i];
                    }
                    uint2 o;
                    o.x = pack_bf16(v[0], v[1]);
                    o.y = pack_bf16(v[2], v[3]);
                    if (RELU) {
                        o.x = relu_bf16x2(o.x);
                        o.y = relu_bf16x2(o.y);
                    }
                    const int pos = (cl >> 3) ^ (r & (CPRW - 1));
                    *reinterpret_cast<uint2 *>(stg + r * STRIP_ROW_BYTES + pos * 16 + ((cl >> 2) & 1) * 8) = o;
                }
            }
#pragma unroll
            for (int j = 0; j < 32 / RPI; ++j) {
                const int rr = j * RPI + lane / CPRW;
                const int ch = lane % CPRW;
                const uint4 val =
                    *reinterpret_cast<const uint4 *>(stg + rr * STRIP_ROW_BYTES + ((ch ^ (rr & (CPRW - 1))) * 16));
                const int row = t.row0 + wm * WTM + mi * 32 + rr;
                const int col = col_base + ch * 8;
                if (row < t.row_end && col < p.N)
                    *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(p.C) + (int64_t)row * p.ldc + col) = val;
            }
        }
    };

    TileInfo t = tile_info(seq);

    if constexpr (KFULL) {
        // ---- global -> LDS without registers: one global_load_lds_dwordx4 moves 64 lanes x 16 B =
        // 1 KB = 8 tile rows into LDS, lane L landing at byte 16*L of the instruction's LDS base.
        // The base is fixed per instruction, so the swizzle is applied on the global side: the lane
        // that lands in chunk slot (L & 7) of row r fetches K chunk (L & 7) ^ ((r >> 1) & 7).
        // Instruction i of wave w fills rows (w*IT + i)*8 .. +7.
        // Per lane: one 64-bit base per operand (row of instruction 0) plus a 32-bit element offset per
        // instruction -- 64-bit pointers per instruction would not fit the register file next to
        // the accumulators of the largest tile.
        const uint16_t *a_base, *b_base;
        int a_off[A_IT], b_off[B_IT];
        auto set_ptrs = [&](const TileInfo &ti) {
            // weights of expert e sit in slot b_slot[e] of the weight array when experts are buffered
            const uint16_t *Bg = Bg0 + (int64_t)((GROUPED && p.b_slot) ? uniform_load(p.b_slot + ti.expert) : ti.expert) * p.strideB;
            int gr0 = 0, gn0 = 0;
#pragma unroll
            for (int i = 0; i < A_IT; ++i) {
                const int r = (wave * A_IT + i) * 8 + (lane >> 3);
                const int kc = (lane & 7) ^ ((r >> 1) & 7);
                int gr = min(ti.row0 + r, ti.row_end - 1);  // rows past the end repeat the last one ...
                if (GROUPED && p.a_zero_row >= 0 && ti.row0 + r >= ti.row_end) gr = p.a_zero_row;  // ... or read zeros
                // dispatch fused into the load: the rows of the expert's batch are gathered straight
                // from the token array (the launcher checked that rows * lda fits 31 bits)
                if (GROUPED && p.a_rows) gr = p.a_rows[gr];
                if (i == 0) {
                    gr0 = gr;
                    a_base = Ag + (int64_t)gr * p.lda + ti.kt0 * BK;
                }
                a_off[i] = (gr - gr0) * (int)p.lda + kc * 8;
            }
            if constexpr (B8) {
                // one instruction = 1 KB = 16 rows of 64 bytes: lane L lands in row (L >> 2), chunk slot
                // (L & 3) and fetches K chunk (L & 3) ^ ((row >> 2) & 3).  In memory that 1 KB block is
                // contiguous and the blocks of a 16-row group follow each other along K (the
                // quantiser's layout), so the offsets are those of the group; they are in bytes,
                // carried as half as many 16-bit units.
                const uint8_t *Bg8 = reinterpret_cast<const uint8_t *>(Bg0) +
                                     (int64_t)((GROUPED && p.b_slot) ? uniform_load(p.b_slot + ti.expert) : ti.expert) * p.strideB;
                const int group_bytes = (K / BK) * 1024;  // one 16-row group over the whole of K
                const int last_group = p.N / 16 - 1;       // groups past the end repeat the last one
#pragma unroll
                for (int i = 0; i < B_IT; ++i) {
                    const int r = (wave * B_IT + i) * 16 + (lane >> 2);
                    const int kc = (lane & 3) ^ ((r >> 2) & 3);
                    const int grp = min((ti.n0 + r) >> 4, last_group);
                    if (i == 0) {
                        gn0 = grp;
                        b_base = reinterpret_cast<const uint16_t *>(Bg8 + (int64_t)grp * group_bytes);
                    }
                    b_off[i] = ((grp - gn0) * group_bytes + (r & 15) * 64 + kc * 16) / 2;
                }
            } else if constexpr (B4) {
                // one instruction = 1 KB = 32 rows of 32 bytes: lane L lands in row (L >> 1), 16-byte half
                // (L & 1); in memory that 1 KB block is contiguous and the blocks of a 32-row group follow
                // each other along K (the quantiser's layout)
                const uint8_t *Bg4 = reinterpret_cast<const uint8_t *>(Bg0) +
                                     (int64_t)((GROUPED && p.b_slot) ? uniform_load(p.b_slot + ti.expert) : ti.expert) * p.strideB;
                const int group_bytes = (K / BK) * 1024;
                const int last_group = p.N / 32 - 1;
#pragma unroll
                for (int i = 0; i < B_IT; ++i) {
                    const int r = (wave * B_IT + i) * 32 + (lane >> 1);
                    const int grp = min((ti.n0 + r) >> 5, last_group);
                    if (i == 0) {
                        gn0 = grp;
                        b_base = reinterpret_cast<const uint16_t *>(Bg4 + (int64_t)grp * group_bytes);
                    }
                    b_off[i] = ((grp - gn0) * group_bytes + (r & 31) * 32 + (lane & 1) * 16) / 2;
                }
            } else {
#pragma unroll
                for (int i = 0; i < B_IT; ++i) {
                    const int r = (wave * B_IT + i) * 8 + (lane >> 3);
                    const int kc = (lane & 7) ^ ((r >> 1) & 7);
                    const int gn = min(ti.n0 + r, p.N - 1);
                    if (i == 0) {
                        gn0 = gn;
                        b_base = Bg + (int64_t)gn * p.ldb + ti.kt0 * BK;
                    }
                    b_off[i] = (gn - gn0) * p.ldb + kc * 8;
                }
            }
        };
        auto issue = [&](int kt, int buf) {
#pragma unroll
            for (int i = 0; i < A_IT; ++i)
                __builtin_amdgcn_global_load_lds((const glb_void *)(a_base + (a_off[i] + kt * BK)),
                                                 (lds_void *)(sA + buf * BM * BK + (wave * A_IT + i) * 8 * BK), 16, 0, 0);
#pragma unroll
            for (int i = 0; i < B_IT; ++i)
                __builtin_amdgcn_global_load_lds((const glb_void *)(b_base + (b_off[i] + kt * (BQ != 0 ? 512 : BK))),
                                                 (lds_void *)(sB + buf * BTILE + (wave * B_IT + i) * 8 * BK), 16, 0, 0);
        };
        // The loads run STAGES-1 K tiles ahead of the MFMAs along the block's whole sequence of
        // (tile, K tile) pairs, so the pipeline never drains between tiles and an epilogue's stores
        // overlap the next tile's first iterations.  Every call issues the same number of loads
        // (past the end of the sequence it re-reads the last K tile into a stage nobody will use),
        // which keeps the vmcnt arithmetic fixed: "at most (STAGES-2) stages' loads outstanding"
        // means the K tile needed next has landed.
        // The barrier between iterations is the bare s_barrier: __syncthreads() would add a full
        // vmcnt(0) wait (it fences the outstanding LDS-bound loads), which serialises the stages.
        // What the barrier must order is covered explicitly: (1) this wave's own global->LDS loads
        // of the stage read next have landed -- the s_waitcnt vmcnt just before it; (2) this
        // wave's LDS reads of the stage overwritten next have returned -- every fragment read is
        // consumed by an MFMA issued before the barrier, and an MFMA does not issue before its
        // operands arrived.
        auto stage_barrier = [&]() {
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
        };
        constexpr int LPS = A_IT + B_IT;             // load instructions per wave per stage
        if constexpr (D16) {
            // ---- 16x16x32 MFMAs out of a ring of K-step slots filled by direct-to-LDS loads.
            // Why 16x16x32: v_mfma_f32_16x16x32_bf16 contracts 32 k per accumulator read and write where
            // v_mfma_f32_32x32x16_bf16 contracts 16; a register-only loop on live data sustains 2.14 PFLOP/s with the
            // former against 1.93 with the latter under the chip's power limit.  Why direct-to-LDS: ds_write_b128 moves
            // 64 bytes per clock per CU (measured) where ds_read_b128 moves 256, so writing a K tile's 64 KB from
            // registers costs the LDS more time than reading its 192 KB of fragments.  Why a ring: a CU takes 64 KB per
            // K tile through a 64-byte-per-clock path -- half the time the MFMAs of that tile need -- so the loads must
            // flow evenly, not in a burst per K tile, and they come from HBM or a remote L2 slice.  With two 64 KB
            // buffers a load can only be issued in the first half of a K tile to land by its end (measured: MFMA pipes
            // 56 % busy; 68 % when every load hits the L2).  Five slots of ONE K step (32 k: 256 + 256 rows of 64 bytes
            // = 32 KB; 160 KB in all) let a wave issue four loads per step, seven MFMAs apart, all the time, each with one to three
            // steps to land: 66 - 73 % busy at a higher clock.
            //
            // Step u multiplies the fragments of slot u mod 5, which were read into registers during step u - 1:
            //   1. the MFMAs of activation block 0 (their operands landed long ago);
            //   2. wait for this wave's LDS reads (all of step u's fragments), on odd steps also for its loads of the
            //      next K tile; barrier.  Behind it every wave's fragments of slot u are in registers, so slots u - 1
            //      and u are free, and the next K tile has landed for everybody;
            //   3. the other MFMAs; behind them the reads of step u + 1's fragments from slot u + 1 (the four weight
            //      fragments into the other register set and block 0 at once, activation block mi in place behind its
            //      last MFMA) and the loads of the K tile two ahead: both halves of a 16-row group back to back (the
            //      second request finds the line in the L1 or merges with the first), the first half into slot u + 4,
            //      the second into slot u + 5 = u.  Loads of a wave land in order, so "at most as many outstanding as
            //      were issued since" is the wait of point 2.
            // A slot row is 64 bytes: 16-byte chunk c of row r sits at position c ^ ((r >> 2) & 3), which keeps the 16
            // lanes x 16 bytes of a fragment read on 16 different bank groups; the permutation is applied on the global
            // side of the load, inside one 64-byte segment.
            // Weight row (output column) permutation inside a wave's columns: LDS row 16 * ni + r holds column
            // 32 * (ni / 2) + 8 * (r / 4) + 4 * (ni % 2) + r % 4, so that the accumulators of blocks 2p and 2p + 1 of a
            // lane are the 8 consecutive columns 32 p + 8 * (lane / 16) ... of token row lane % 16 and leave as one
            // 16-byte store, without a trip through LDS (all of which the ring holds).
            static_assert(GROUPED, "the ring pipeline is instantiated for the grouped GEMM");
            constexpr int NSLOT = 5;
            constexpr int SLOT_BYTES = (BM + BN) * 64;
            constexpr int MI16 = WTM / 16, NI16 = WTN / 16;
            constexpr int NWAVE = THREADS / 64;
            constexpr int AG = BM / 16 / NWAVE, BG = BN / 16 / NWAVE;  // 16-row groups a wave loads per K tile
            constexpr int PAIRS = AG + BG;
            constexpr int Q1 = PAIRS / 2;                              // pairs issued in the even step; the rest in the odd one
            constexpr int PB = 1;                                      // activation blocks multiplied in front of the barrier
            constexpr int PRE = PB * NI16;
            constexpr int NM16 = MI16 * NI16;
            constexpr bool ACC16_IN_AGPR = NM16 * 4 > 128;
            static_assert(BM % (16 * NWAVE) == 0 && BN % (16 * NWAVE) == 0 && WTN % 32 == 0 && MI16 >= 2 && PB < MI16 - 1, "ring pipeline tile shape");
            static_assert(BK == 64, "a K tile is two steps of 32");
            f32x4 acc16[MI16][NI16];
            const int wave_u = __builtin_amdgcn_readfirstlane(wave);
            const int row16 = lane & 15, kq = lane >> 4;
            // fragment reads: row (block base + row16), chunk position kq ^ ((row16 >> 2) & 3)
            const int frag_off = row16 * 64 + ((kq ^ ((row16 >> 2) & 3)) << 4);
            const uint8_t *fragA = smem_raw + (wm * WTM) * 64 + frag_off;
            const uint8_t *fragB = smem_raw + BM * 64 + (wn * WTN) * 64 + frag_off;
            // load stream
            int l_seq = seq, l_kt = 0;
            bool l_more = true;
            int w_slot = 0;  // slot of the first half of the K tile the stream is at
            const uint8_t *srcA, *srcB;  // same for every lane: the operand's first byte of the stream's K tile
            uint32_t a_voff[AG][2], b_voff[BG][2];
            const int ld_row = lane >> 2;                              // row inside the 16-row group
            const int ld_chunk = (lane & 3) ^ ((lane >> 4) & 3);      // K chunk this lane fetches for its LDS position
            auto set_ptrs16 = [&](const TileInfo &ti) {
                const int slot = p.b_slot ? uniform_load(p.b_slot + ti.expert) : ti.expert;
                srcB = reinterpret_cast<const uint8_t *>(Bg0 + (int64_t)slot * p.strideB);
                srcA = reinterpret_cast<const uint8_t *>(Ag);
#pragma unroll
                for (int g = 0; g < AG; ++g) {
                    const int r = (wave * AG + g) * 16 + ld_row;
                    int gr = min(ti.row0 + r, ti.row_end - 1);
                    if (p.a_zero_row >= 0 && ti.row0 + r >= ti.row_end) gr = p.a_zero_row;
                    if (p.a_rows) gr = p.a_rows[gr];
                    const uint32_t o = (uint32_t)gr * (uint32_t)p.lda * 2u + ld_chunk * 16;
                    a_voff[g][0] = o;
                    a_voff[g][1] = o + 64;
                }
#pragma unroll
                for (int g = 0; g < BG; ++g) {
                    const int rho = (wave * BG + g) * 16 + ld_row;  // LDS row of the tile
                    const int x = rho % WTN, xi = x >> 4, xr = x & 15;
                    const int c = (rho / WTN) * WTN + 32 * (xi >> 1) + 8 * (xr >> 2) + 4 * (xi & 1) + (xr & 3);
                    const int gn = min(ti.n0 + c, p.N - 1);
                    const uint32_t o = (uint32_t)gn * (uint32_t)p.ldb * 2u + ld_chunk * 16;
                    b_voff[g][0] = o;
                    b_voff[g][1] = o + 64;
                }
            };
            auto issue_load = [&](int j) {  // load j of the stream's K tile: pair j / 2, K half j % 2
                const int g = j >> 1, h = j & 1;
                int slot = w_slot + h;
                if (slot >= NSLOT) slot -= NSLOT;
                if (g < AG)
                    __builtin_amdgcn_global_load_lds((const glb_void *)(srcA + (size_t)l_kt * 128 + a_voff[g][h]),
                                                     (lds_void *)(smem_raw + slot * SLOT_BYTES + (wave_u * AG + g) * 1024), 16, 0, 0);
                else
                    __builtin_amdgcn_global_load_lds((const glb_void *)(srcB + (size_t)l_kt * 128 + b_voff[g - AG][h]),
                                                     (lds_void *)(smem_raw + slot * SLOT_BYTES + BM * 64 + (wave_u * BG + (g - AG)) * 1024), 16, 0, 0);
            };
            auto advance = [&]() {
                w_slot += 2;
                if (w_slot >= NSLOT) w_slot -= NSLOT;
                if (l_more && ++l_kt == KT) {
                    if (seq_ok(l_seq + slots)) {
                        l_seq += slots;
                        l_kt = 0;
                        set_ptrs16(tile_info(l_seq));
                    } else {
                        l_more = false;
                        l_kt = KT - 1;  // past the end: re-read the last K tile into slots nobody reads
                    }
                }
            };
            // a16[MI16 - 1 + P]: the last activation block has a register set per step parity, so that its read for the
            // next step goes out with the first ones and the step's last LDS read is four MFMAs from the step's end
            bf16x8 a16[MI16 + 1], w16[2][NI16];
            int r_slot = 0;  // slot of the step being multiplied
            auto read_frag = [&](const uint8_t *base, int slot, int block) {
                return *reinterpret_cast<const bf16x8 *>(base + slot * SLOT_BYTES + block * 1024);
            };
            auto step = [&](auto parity) {
                constexpr int P = decltype(parity)::value;
                constexpr int NL = P == 0 ? 2 * Q1 : 2 * (PAIRS - Q1);  // loads issued in this step
                constexpr int J0 = P == 0 ? 0 : 2 * Q1;
                constexpr int GAP = NL > 0 ? ((NM16 - PRE) / NL > 8 ? 8 : (NM16 - PRE) / NL) : 1;  // MFMAs between two loads
                static_assert(NL == 0 || GAP >= 1, "more loads than MFMA slots behind the barrier");
                auto mfma = [&](int mi, int ni) {
                    acc16[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w16[P][ni], a16[mi == MI16 - 1 ? mi + P : mi], acc16[mi][ni], 0, 0, 0);
                };
#pragma unroll
                for (int mi = 0; mi < PB; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NI16; ++ni) mfma(mi, ni);
                __builtin_amdgcn_sched_barrier(0);
                asm volatile("" ::: "memory");
                // lgkmcnt(0); odd steps: at most the loads of the even step before may be outstanding
                if (P == 1)
                    __builtin_amdgcn_s_waitcnt(0x0070 | ((2 * Q1) & 15) | (((2 * Q1) >> 4) << 14));
                else
                    __builtin_amdgcn_s_waitcnt(0xc07f);
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
                const int nslot = r_slot + 1 == NSLOT ? 0 : r_slot + 1;
#pragma unroll
                for (int ni = 0; ni < NI16; ++ni) w16[P ^ 1][ni] = read_frag(fragB, nslot, ni);
#pragma unroll
                for (int mi = 0; mi < PB; ++mi) a16[mi] = read_frag(fragA, nslot, mi);
                a16[MI16 - 1 + (P ^ 1)] = read_frag(fragA, nslot, MI16 - 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int mi = PB; mi < MI16; ++mi) {
#pragma unroll
                    for (int ni = 0; ni < NI16; ++ni) {
                        const int gm = mi * NI16 + ni;
                        mfma(mi, ni);
                        if (ni == NI16 - 1 && mi < MI16 - 1) a16[mi] = read_frag(fragA, nslot, mi);
                        if (NL > 0 && (gm - PRE) % GAP == 0 && (gm - PRE) / GAP < NL) issue_load(J0 + (gm - PRE) / GAP);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                r_slot = nslot;
                if (P == (Q1 == PAIRS ? 0 : 1)) advance();  // behind the K tile's last load
                __builtin_amdgcn_sched_barrier(0);
            };
            auto epilogue16 = [&](const TileInfo &ti) {
                const uint16_t *bias = static_cast<const uint16_t *>(p.bias);
                if (bias) bias += (int64_t)ti.expert * p.strideBias;
                const int col_base = ti.n0 + wn * WTN + 8 * kq;
                uint8_t *const cbase = static_cast<uint8_t *>(p.C);
                const uint32_t row_step = 16u * (uint32_t)p.ldc * 2u;  // bytes between two row blocks
                auto store_all = [&](auto with_bias) {
                    constexpr bool BIAS = decltype(with_bias)::value;
                    uint32_t bw[NI16 / 2][4] = {};
                    if constexpr (BIAS) {
#pragma unroll
                        for (int pp = 0; pp < NI16 / 2; ++pp)
                            if (col_base + 32 * pp < p.N) {  // N is a multiple of 8
                                const uint4 bb = *reinterpret_cast<const uint4 *>(bias + col_base + 32 * pp);
                                bw[pp][0] = bb.x, bw[pp][1] = bb.y, bw[pp][2] = bb.z, bw[pp][3] = bb.w;
                            }
                    }
                    const int row0 = ti.row0 + wm * WTM + row16;
                    uint32_t off = (uint32_t)row0 * (uint32_t)p.ldc * 2u + (uint32_t)col_base * 2u;  // the launcher checked that C fits 32 bits
#pragma unroll
                    for (int mi = 0; mi < MI16; ++mi) {
                        // the column pairs of a row block back to back: together they fill whole 128-byte lines
#pragma unroll
                        for (int pp = 0; pp < NI16 / 2; ++pp) {
                            uint32_t o[4];
#pragma unroll
                            for (int q = 0; q < 4; ++q) {  // columns 2q, 2q + 1 of the 8: block 2pp + q / 2, registers 2 (q % 2), + 1
                                float v0, v1;
                                if constexpr (ACC16_IN_AGPR) {  // read in place, as in the 32x32 epilogue
                                    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v0) : "a"(acc16[mi][2 * pp + (q >> 1)][2 * (q & 1)]));
                                    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v1) : "a"(acc16[mi][2 * pp + (q >> 1)][2 * (q & 1) + 1]));
                                } else {
                                    v0 = acc16[mi][2 * pp + (q >> 1)][2 * (q & 1)], v1 = acc16[mi][2 * pp + (q >> 1)][2 * (q & 1) + 1];
                                }
                                if constexpr (BIAS) {
                                    v0 += __uint_as_float(bw[pp][q] << 16);
                                    v1 += __uint_as_float(bw[pp][q] & 0xffff0000u);
                                }
                                o[q] = pack_bf16(v0, v1);
                                if (RELU) o[q] = relu_bf16x2(o[q]);
                            }
                            if (row0 + mi * 16 < ti.row_end && col_base + 32 * pp < p.N)
                                *reinterpret_cast<uint4 *>(cbase + off + 64 * pp) = make_uint4(o[0], o[1], o[2], o[3]);
                        }
                        off += row_step;
                    }
                };
                if constexpr (ACC16_IN_AGPR) asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
                if (bias)
                    store_all(std::true_type{});
                else
                    store_all(std::false_type{});
            };
            // prologue: the first two K tiles of the stream -> slots 0..3; fragments of step 0
            set_ptrs16(t);
#pragma unroll
            for (int rep = 0; rep < 2; ++rep) {
#pragma unroll
                for (int j = 0; j < 2 * PAIRS; ++j) issue_load(j);
                advance();
            }
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_waitcnt(0x0f70 | ((2 * PAIRS) & 15) | (((2 * PAIRS) >> 4) << 14));  // the first K tile has landed
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ni = 0; ni < NI16; ++ni) w16[0][ni] = read_frag(fragB, 0, ni);
#pragma unroll
            for (int mi = 0; mi < MI16; ++mi) a16[mi] = read_frag(fragA, 0, mi);  // step 0 is even: its last block is a16[MI16 - 1]
            while (true) {
#pragma unroll
                for (int mi = 0; mi < MI16; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NI16; ++ni)
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc16[mi][ni][r] = 0.f;
                for (int kt = 0; kt < KT; ++kt) {
                    step(std::integral_constant<int, 0>{});
                    step(std::integral_constant<int, 1>{});
                }
                epilogue16(t);
                seq += slots;
                if (!seq_ok(seq)) break;
                t = tile_info(seq);
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no LDS write may outlive the block
            return;
        }
        if constexpr (RSTAGE) {
            // ---- register-staged pipeline.  A vector-memory instruction costs the issuing wave
            // about one MFMA slot and the CU's address unit 16 clocks, so the loads of a K tile
            // must neither come as one burst (every wave stalls in the queue while the matrix
            // units idle) nor late (two LDS buffers leave no slack for their latency).  Here the
            // LPS loads of K tile i+2 go into registers, one behind every (MFMAs per K tile / LPS)-th
            // MFMA of iteration i; one iteration later, at the same slot, the register is written
            // to the LDS buffer of tile i+1 (ds_write_b128, 1 KB contiguous per wave instruction)
            // and immediately refilled.  Every load has a whole iteration to land, the address unit
            // sees an even stream, and the LDS buffer written in an iteration is the one nobody
            // reads until the barrier that ends it.
            constexpr int KS = BK / 16, NM = MI * NI, NR = MI + NI, TM = KS * NM;
            int l_seq = seq, l_kt = 0;
            bool l_more = true;
            set_ptrs(t);
            uint4 R[LPS];
            auto gload = [&](int i) -> uint4 {
                const uint16_t *g = i < A_IT ? a_base + (a_off[i] + l_kt * BK) : b_base + (b_off[i - A_IT] + l_kt * BK);
                return *reinterpret_cast<const uint4 *>(g);
            };
            auto lds_put = [&](int buf, int i, const uint4 &v) {
                uint16_t *d = i < A_IT ? sA + buf * BM * BK + (wave * A_IT + i) * 8 * BK
                                       : sB + buf * BTILE + (wave * B_IT + (i - A_IT)) * 8 * BK;
                *reinterpret_cast<uint4 *>(d + lane * 8) = v;
            };
            auto advance = [&]() {
                if (l_more && ++l_kt == KT) {
                    if (seq_ok(l_seq + slots)) {
                        l_seq += slots;
                        l_kt = 0;
                        set_ptrs(tile_info(l_seq));
                    } else {
                        l_more = false;
                        l_kt = KT - 1;  // past the end: re-read the last K tile, never used
                    }
                }
            };
            bf16x8 af[2][MI], bfr[2][NI];
            auto read_one = [&](int buf, int ks, int set, int m) {
                const int chunkpos = ((ks * 2 + frag_half) ^ swz) << 3;
                if (m < MI)
                    af[set][m] = *reinterpret_cast<const bf16x8 *>(sA + buf * BM * BK + (wm * WTM + frag_row + m * 32) * BK +
                                                                   chunkpos);
                else
                    bfr[set][m - MI] = *reinterpret_cast<const bf16x8 *>(
                        sB + buf * BTILE + (wn * WTN + frag_row + (m - MI) * 32) * BK + chunkpos);
            };
            // the ds_writes of this iteration must be complete before anyone reads the buffer
            auto rs_sync = [&]() {
                __builtin_amdgcn_sched_barrier(0);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
            };
            // One K tile out of LDS buffer cur; the instruction order is pinned MFMA by MFMA.
            auto compute_rs = [&](int cur) {
                const int nxt = cur ^ 1;
#pragma unroll
                for (int m = 0; m < NR; ++m) read_one(cur, 0, 0, m);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                    for (int m = 0; m < NM; ++m) {
                        if (ks + 1 < KS) {  // fragment f of the next K-step is read behind MFMA f * NM / NR
#pragma unroll
                            for (int f = 0; f < NR; ++f)
                                if (f * NM / NR == m) read_one(cur, ks + 1, (ks + 1) & 1, f);
                        }
                        const int mi = m / NI, ni = m % NI;
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ks & 1][ni], af[ks & 1][mi],
                                                                              acc[mi][ni], 0, 0, 0);
                        const int gm = ks * NM + m;
#pragma unroll
                        for (int i = 0; i < LPS; ++i) {
                            if ((i * TM + TM / 2) / LPS == gm) {  // slot i sits behind MFMA number (i + 1/2) * TM / LPS
                                lds_put(nxt, i, R[i]);
                                R[i] = gload(i);
                            }
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                advance();
                rs_sync();
            };
            // prologue: K tile 0 -> LDS buffer 0, K tile 1 -> registers
#pragma unroll
            for (int i = 0; i < LPS; ++i) R[i] = gload(i);
            advance();
#pragma unroll
            for (int i = 0; i < LPS; ++i) lds_put(0, i, R[i]);
#pragma unroll
            for (int i = 0; i < LPS; ++i) R[i] = gload(i);
            advance();
            rs_sync();
            // (Letting the waves whose rows all lie past the end of an expert's batch skip their MFMAs
            // makes such a tile 13 % shorter, but the CUs of an XCD then drift apart, share less of the
            // weight panels in L2, and the launch fetches 45 % more from HBM: slower overall.)
            int cur = 0;
            while (true) {
                zero_acc();
                for (int kt = 0; kt < KT; ++kt) {
                    compute_rs(cur);
                    cur ^= 1;
                }
                if constexpr (LDS_EPILOGUE)
                    epilogue_lds(t, cur ^ 1);  // the buffer the last K tile was read from
                else
                    epilogue(t);
                seq += slots;
                if (!seq_ok(seq)) break;
                t = tile_info(seq);
            }
            return;
        }
        constexpr int WAITN = STAGES >= 2 ? (STAGES - 2) * LPS : 0;
        // s_waitcnt vmcnt(WAITN), through the builtin and not as inline assembly: the compiler's own wait-count
        // bookkeeping reads the builtin and then knows that every older load has landed.  It cannot see into
        // inline assembly; with that, a register load left over from an epilogue counted as still in flight
        // and the compiler drained the whole load pipeline (vmcnt(0)) at the top of every K iteration.
        // Encoding: vmcnt in bits 3:0 and 15:14, expcnt (bits 6:4) and lgkmcnt (bits 11:8) left at "no wait".
        auto wait_loads = [&]() {
            static_assert(WAITN >= 0 && WAITN < 64, "vmcnt is a 6-bit counter");
            constexpr int kWaitImm = (WAITN & 15) | ((WAITN >> 4) << 14) | (7 << 4) | (15 << 8);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_waitcnt(kWaitImm);
            asm volatile("" ::: "memory");
        };
        int l_seq = seq, l_kt = 0, l_stage = 0;
        bool l_more = true;
        set_ptrs(t);
        auto issue_next = [&]() {
            issue(l_kt, l_stage);
            l_stage = (l_stage + 1 == STAGES) ? 0 : l_stage + 1;
            if (l_more && ++l_kt == KT) {
                if (seq_ok(l_seq + slots)) {
                    l_seq += slots;
                    l_kt = 0;
                    set_ptrs(tile_info(l_seq));
                } else {
                    l_more = false;
                    l_kt = KT - 1;
                }
            }
        };
        // 4-bit weights: the scale bytes run one group of 8 K tiles ahead of the MFMAs, across tile borders.
        // One load instruction per wave fills 64 rows x 16 bytes of the buffer: lane L fetches the 16 bytes
        // of row 64 * wave + L (row group 2 * wave + L / 32 of the tile, row L % 32 of that group's 512-byte
        // block).  These loads are older than the operand loads issued after them, and loads complete in
        // order, so the per-iteration vmcnt wait covers them once two iterations have passed.
        int s_seq = seq, s_grp = 0, s_buf = 0;
        const uint8_t *s_lane = nullptr;
        const int s_groups = (KT + 7) >> 3;  // 16-byte scale groups per weight row
        auto scale_tile = [&]() {
            const TileInfo ts = tile_info(s_seq);
            const int rg = min((ts.n0 + wave * 64 + (lane >> 5) * 32) >> 5, p.N / 32 - 1);
            s_lane = p.b_blk_scale + (int64_t)ts.expert * p.stride_blk_scale + (int64_t)rg * s_groups * 512 + (lane & 31) * 16;
        };
        auto issue_scales = [&]() {
            if constexpr (B4) {
                __builtin_amdgcn_global_load_lds((const glb_void *)(s_lane + s_grp * 512),
                                                 (lds_void *)(sS + s_buf * (BN * 16) + wave * 1024), 16, 0, 0);
                s_buf ^= 1;
                if (++s_grp == s_groups) {  // on to the next tile of this block, if there is one
                    s_grp = 0;
                    if (seq_ok(s_seq + slots)) {
                        s_seq += slots;
                        scale_tile();
                    }
                }
            }
        };
        if constexpr (B4) {
            scale_tile();
            issue_scales();
            issue_scales();
        }
#pragma unroll
        for (int i = 0; i < STAGES - 1; ++i) issue_next();
        wait_loads();
        stage_barrier();
        int stage = 0;
        while (true) {
            zero_acc();
            for (int kt = 0; kt < KT; ++kt) {
                if constexpr (B4) {
                    if ((kt & 7) == 0 && (kt > 0 || seq != (int)(blockIdx.x >> 3))) {  // a new group of 8 K tiles
                        if (KT < STAGES) {
                            // groups shorter than the pipeline is deep: the scales requested one group ago
                            // may not have landed yet
                            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                            stage_barrier();
                        }
                        c_buf ^= 1;
                        issue_scales();  // into the buffer of the group just finished
                    }
                }
                issue_next();  // into the stage the previous iteration computed from
                compute(stage, kt);
                wait_loads();
                stage_barrier();
                stage = (stage + 1 == STAGES) ? 0 : stage + 1;
            }
            if constexpr (LDS_EPILOGUE)
                epilogue_lds(t, stage == 0 ? STAGES - 1 : stage - 1);  // the stage the last K tile was read from
            else
                epilogue(t);
            seq += slots;
            if (!seq_ok(seq)) break;
            t = tile_info(seq);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no LDS write may outlive the block
    } else {
        // ---- K not a multiple of the K tile: stage through registers so the tail can be zero filled.
        // chunk c = tid + i*THREADS; row = c >> 3, kc = c & 7
        const int kc = tid & 7;
        while (true) {
            const uint16_t *Bg = Bg0 + (int64_t)((GROUPED && p.b_slot) ? uniform_load(p.b_slot + t.expert) : t.expert) * p.strideB;
            const uint16_t *a_ptr[A_IT];
            const uint16_t *b_ptr[B_IT];
            int a_lds[A_IT], b_lds[B_IT];
#pragma unroll
            for (int i = 0; i < A_IT; ++i) {
                const int r = (tid + i * THREADS) >> 3;
                const int gr = min(t.row0 + r, t.row_end - 1);
                a_ptr[i] = Ag + (int64_t)gr * p.lda + kc * 8;
                a_lds[i] = r * BK + ((kc ^ ((r >> 1) & 7)) << 3);
            }
#pragma unroll
            for (int i = 0; i < B_IT; ++i) {
                const int r = (tid + i * THREADS) >> 3;
                const int gn = min(t.n0 + r, p.N - 1);
                b_ptr[i] = Bg + (int64_t)gn * p.ldb + kc * 8;
                b_lds[i] = r * BK + ((kc ^ ((r >> 1) & 7)) << 3);
            }
            uint4 a_reg[A_IT], b_reg[B_IT];
            auto load_global = [&](int kt) {
                const int k0 = kt * BK;
                const bool ok = k0 + kc * 8 < K;
#pragma unroll
                for (int i = 0; i < A_IT; ++i)
                    a_reg[i] = ok ? *reinterpret_cast<const uint4 *>(a_ptr[i] + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
                for (int i = 0; i < B_IT; ++i)
                    b_reg[i] = ok ? *reinterpret_cast<const uint4 *>(b_ptr[i] + k0) : make_uint4(0, 0, 0, 0);
            };
            auto store_lds = [&](int buf) {
#pragma unroll
                for (int i = 0; i < A_IT; ++i) *reinterpret_cast<uint4 *>(sA + buf * BM * BK + a_lds[i]) = a_reg[i];
#pragma unroll
                for (int i = 0; i < B_IT; ++i) *reinterpret_cast<uint4 *>(sB + buf * BN * BK + b_lds[i]) = b_reg[i];
            };
            zero_acc();
            load_global(0);
            store_lds(0);
            __syncthreads();
            for (int kt = 0; kt < KT; ++kt) {
                const int cur = kt & 1;
                if (kt + 1 < KT) load_global(kt + 1);
                compute(cur, kt);
                if (kt + 1 < KT) store_lds(cur ^ 1);
                __syncthreads();
            }
            epilogue(t);
            seq += slots;
            if (!seq_ok(seq)) break;
            t = tile_info(seq);
        }
    }
}

template <int BM, int BN, int WM, int WN, bool OUT_F32, bool RELU, bool GROUPED, bool KFULL, int MINB, int STAGES,
          int BQ = 0>
static int launch_k(const GemmParams &p_in, int num_cus, hipStream_t s, int *main_grid)
{
    GemmParams p = p_in;
    const int n_tiles = ceil_div(p.N, BN);
    const int m_tiles = GROUPED ? p.max_m_tiles : ceil_div(p.M, BM);
    if (m_tiles <= 0 || n_tiles <= 0) return MOE_OK;
    const size_t smem = STAGES == DTL16 ? (size_t)5 * (BM + BN) * 64  // five slots of one 32-wide K step
                                        : (size_t)(STAGES == REG_STAGED ? 2 : STAGES) * (BM + (BQ == 8 ? BN / 2 : BQ == 4 ? BN / 4 : BN)) * BK * sizeof(uint16_t) +
                                              (BQ == 4 ? 2 * BN * 16 : 0);  // 4-bit weights: two buffers of block scales
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN, OUT_F32, RELU, GROUPED, KFULL, MINB, STAGES, BQ>;
    // per instantiation, once, whichever host thread comes first: the LDS size attribute and the occupancy
    static std::once_flag once;
    static int blocks_per_cu = 0;
    static hipError_t setup_rc = hipSuccess;
    std::call_once(once, [&]() {
        setup_rc = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)smem);
        int occ = 0;
        if (setup_rc == hipSuccess) setup_rc = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kern, WM * WN * 64, smem);
        blocks_per_cu = occ < 1 ? 1 : (occ > 8 ? 8 : occ);
    });
    MOE_HIP_CHECK(setup_rc);
    // persistent grid: every resident slot of the chip, but never more blocks than upper-bound tiles
    int64_t grid = (int64_t)num_cus * blocks_per_cu;
    int64_t tiles = (int64_t)m_tiles * n_tiles;
    if (!GROUPED && p.k_split > 1) {
        if (!KFULL || (p.K / BK) % p.k_split != 0) {
            set_error("split K: %d does not divide the %d K tiles", p.k_split, p.K / BK);
            return MOE_ERR_INVALID_ARG;
        }
        tiles *= p.k_split;
    }
    if (p.tail_mode == 2) {
        // max_m_tiles counts 256-row parents; at most (main_slots * 5 - 1) / 9 of the parent tiles are left over
        p.main_slots = *main_grid;
        const int64_t parents = (int64_t)m_tiles * ceil_div(p.N, 256);
        const int64_t left_max = ((int64_t)p.main_slots * 5 - 1) / 9;
        tiles = (parents < left_max ? parents : left_max) * ((256 / BM) * (256 / BN));
        if (tiles <= 0) return MOE_OK;
    }
    if (grid > tiles) grid = tiles;
    grid = align_up(grid, 8);
    if (p.tail_mode == 1) {
        p.main_slots = (int)grid;
        *main_grid = (int)grid;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(WM * WN * 64), smem, s, p);
    MOE_LAUNCH_CHECK("gemm_bf16_kernel");
    return MOE_OK;
}

template <int BM, int BN, int WM, int WN, bool OUT_F32, bool RELU, bool GROUPED, int MINB, int STAGES = 2>
static int launch_one(const GemmParams &p, int num_cus, hipStream_t s, int *main_grid = nullptr)
{
    // K a multiple of the K tile: pipelined main loop without a tail predicate; the K-tail path
    // always uses two LDS stages
    return (p.K % BK == 0)
               ? launch_k<BM, BN, WM, WN, OUT_F32, RELU, GROUPED, true, MINB, STAGES>(p, num_cus, s, main_grid)
               : launch_k<BM, BN, WM, WN, OUT_F32, RELU, GROUPED, false, MINB, 2>(p, num_cus, s, main_grid);
}

// grouped GEMM with 8-bit (BQ = 8) or 4-bit (BQ = 4) weights (K a multiple of the K tile: checked by the caller)
template <int BM, int BN, int WM, int WN, int MINB, int STAGES, int BQ = 8>
static int launch_grouped_w8(const GemmParams &p, bool relu, int num_cus, hipStream_t s)
{
    return relu ? launch_k<BM, BN, WM, WN, false, true, true, true, MINB, STAGES, BQ>(p, num_cus, s, nullptr)
                : launch_k<BM, BN, WM, WN, false, false, true, true, MINB, STAGES, BQ>(p, num_cus, s, nullptr);
}

// Tile shapes of the grouped GEMM.  variant -> (BM, BN, waves, pipeline)
//   8: 256x256, 8 waves, register-staged    10: 128x128, 4 waves, register-staged
//   2: 64x128, 4 waves, direct-to-LDS        3: 32x128, 4 waves, direct-to-LDS
// The choice goes by the average number of rows per expert.  (Direct-to-LDS forms of the two large shapes
// measured 7-8 % slower than the register-staged ones; a 128x256 shape, meant to quantise better over the
// CUs when a GEMM has only one or two 256x256 tiles per CU, measured 16 % slower per flop and lost even there.)
// every grouped bf16 shape reads A through per-lane row pointers when K is a multiple of the K tile
bool gemm_bf16_variant_gathers(int variant, int K) { return variant != 0 && K % BK == 0; }

// 8-bit weights are for the weight-streaming regime: always the small tiles (three / four LDS
// stages deep, the stages cost half the LDS), whatever the row count.  (Measured on 128 experts of
// 2048 x 8192 with 1 to 64 rows each: 2 to 6 stages, 32x64 and 32x256 tiles and up to 6 blocks per
// CU all land within +-8 % of these two; deeper pipelines lose blocks per CU and are slower.)
int gemm_bf16_variant_w8(int64_t n_rows, int E)
{
    const int64_t avg = E > 0 ? n_rows / E : n_rows;
    return avg >= 48 ? 22 : 23;
}

// 4-bit weights: 43 = 32x256, 48 = 64x256, three LDS stages each plus the two scale buffers (32x256: 44 KB,
// three blocks per CU; a fourth stage would leave room for two, 0.141 -> 0.154 ms on the decoder's first
// GEMM; two stages 0.150).  (Measured on 128 experts of 2048 x 8192
// with 1 to 64 rows each: 256 columns per tile beat 128 by 25-30 % -- the A tile, re-read once per column
// tile, weighs as much as a 128-column B tile at 4 bits -- and 512 lost again.
// With 8 or 16 tokens the second GEMM has fewer tiles than CUs and its time is the K loop of one tile,
// 128 K tiles at about 0.65 us each, whatever the tile width or pipeline depth: only a split along K
// would shorten it.)
int gemm_bf16_variant_w4(int64_t n_rows, int E)
{
    const int64_t avg = E > 0 ? n_rows / E : n_rows;
    return avg >= 96 ? 48 : 43;
}

// K ranges for the fp32-output plain GEMM (the gate): 1 unless the 32-row tiles would leave most of the
// chip idle; then the largest power of two <= 16 that divides the K tile count, keeps two K tiles per
// range and does not make more tiles than CUs.
int gemm_bf16_gate_split(int M, int N, int K, int num_cus)
{
    if (K % BK != 0) return 1;
    const int bn = N <= 32 ? 32 : (N <= 64 ? 64 : 128);
    const int64_t tiles = (int64_t)ceil_div(M, 32) * ceil_div(N, bn);
    if ((int64_t)ceil_div(M, 128) * ceil_div(N, 128) >= 2 * (int64_t)num_cus) return 1;  // the 128-row shape runs
    const int kt = K / BK;
    int s = 1;
    while (s * 2 <= 16 && kt % (s * 2) == 0 && kt / (s * 2) >= 2 && tiles * s * 2 <= num_cus) s *= 2;
    return s;
}

int gemm_bf16_variant_block_m(int v)
{
    switch (v) {
    case 10: return 128;
    case 2: case 22: case 48: return 64;
    case 3: case 23: case 43: return 32;
    default: return 256;
    }
}

int gemm_bf16_variant(int64_t n_rows, int E, int N, int num_cus)
{
    (void)N;
    (void)num_cus;
    const int64_t avg = E > 0 ? n_rows / E : n_rows;
    if (avg >= 192) return 8;
    if (avg >= 96) return 10;
    if (avg >= 48) return 2;
    return 3;
}

template <int BM, int BN, int WM, int WN, int MINB, int STAGES = 2>
static int launch_grouped(const GemmParams &p, bool relu, int num_cus, hipStream_t s, int *main_grid = nullptr)
{
    return relu ? launch_one<BM, BN, WM, WN, false, true, true, MINB, STAGES>(p, num_cus, s, main_grid)
                : launch_one<BM, BN, WM, WN, false, false, true, MINB, STAGES>(p, num_cus, s, main_grid);
}

// Dispatch over the instantiated shapes.
int launch_gemm_bf16(const GemmParams &p, bool grouped, int variant, bool out_f32, bool relu, int num_cus,
                     hipStream_t s)
{
    if (!grouped) {
        // gate: fp32 logits, N = E is small
        if (relu) {
            set_error("plain bf16 GEMM is not instantiated with ReLU");
            return MOE_ERR_UNSUPPORTED;
        }
        // bf16 output: the dense mask multiplications of the static-capacity baseline
        if (!out_f32) return launch_one<256, 256, 2, 4, false, false, false, 1, REG_STAGED>(p, num_cus, s);
        // 128-row tiles when they still fill the chip twice over, else 32-row tiles: the K loop of such a
        // skinny GEMM is latency bound, so the number of tiles in flight is what streams x
        const bool tall = (int64_t)ceil_div(p.M, 128) * ceil_div(p.N, 128) >= 2 * (int64_t)num_cus;
        // 32-row tiles run four LDS stages deep (three K tiles in flight per block)
        if (p.N <= 32)
            return tall ? launch_one<128, 32, 4, 1, true, false, false, 2>(p, num_cus, s)
                        : launch_one<32, 32, 1, 1, true, false, false, 2, 4>(p, num_cus, s);
        if (p.N <= 64)
            return tall ? launch_one<128, 64, 2, 2, true, false, false, 2>(p, num_cus, s)
                        : launch_one<32, 64, 1, 2, true, false, false, 2, 4>(p, num_cus, s);
        return tall ? launch_one<128, 128, 2, 2, true, false, false, 2>(p, num_cus, s)
                    : launch_one<32, 128, 1, 4, true, false, false, 2, 4>(p, num_cus, s);
    }
    if (out_f32) {
        set_error("grouped bf16 GEMM is only instantiated for bf16 output");
        return MOE_ERR_UNSUPPORTED;
    }
    switch (variant) {
    case 8: {
        // whole rounds as 256x256 tiles, the partly filled last round as 128x128 sub-tiles
        if (p.K % BK != 0) return launch_grouped<256, 256, 2, 4, 1, REG_STAGED>(p, relu, num_cus, s);
        GemmParams q = p;
        int main_grid = 0;
        q.tail_mode = 1;
        // the ring pipeline addresses both operands with 32-bit byte offsets from one base
        const int64_t a_rows_max = (int64_t)(p.a_zero_row >= p.M ? p.a_zero_row + 1 : p.M);
        const bool ring_ok = a_rows_max * p.lda * 2 < (1ll << 32) && (int64_t)p.N * p.ldb * 2 < (1ll << 32) &&
                             ((int64_t)(p.c_zero_row >= p.M ? p.c_zero_row + 1 : p.M) + 256) * p.ldc * 2 < (1ll << 32);
        int rc = ring_ok ? launch_grouped<256, 256, 2, 4, 1, DTL16>(q, relu, num_cus, s, &main_grid)
                         : launch_grouped<256, 256, 2, 4, 1, REG_STAGED>(q, relu, num_cus, s, &main_grid);
        if (rc != MOE_OK || main_grid == 0) return rc;
        q.tail_mode = 2;
        return launch_grouped<128, 128, 2, 2, 2, REG_STAGED>(q, relu, num_cus, s, &main_grid);
    }
    case 10: return launch_grouped<128, 128, 2, 2, 2, REG_STAGED>(p, relu, num_cus, s);
    case 22: return launch_grouped_w8<64, 128, 1, 4, 2, 3>(p, relu, num_cus, s);
    case 23: return launch_grouped_w8<32, 128, 1, 4, 2, 4>(p, relu, num_cus, s);
    case 43: return launch_grouped_w8<32, 256, 1, 4, 2, 3, 4>(p, relu, num_cus, s);
    case 48: return launch_grouped_w8<64, 256, 1, 4, 2, 3, 4>(p, relu, num_cus, s);
    case 2: return launch_grouped<64, 128, 1, 4, 2>(p, relu, num_cus, s);
    case 3: return launch_grouped<32, 128, 1, 4, 2>(p, relu, num_cus, s);
    default:
        set_error("unsupported grouped GEMM variant %d", variant);
        return MOE_ERR_UNSUPPORTED;
    }
}

}  // namespace moe355
