// Projections of the verify step: out[T, N] = X[T, K] * W[N, K]^T over the packed rows of a batch.
//
// bf16 path (the one that matters): T is about 100-600 packed rows, so every weight byte is used
// for only T multiply-adds and the kernel is a weight stream bounded by HBM.  It is still a dense
// contraction, so the arithmetic goes through v_mfma_f32_32x32x16_bf16 (the 16x16 shapes run at
// about half its rate on gfx950, which would make them, not HBM, the bound).
//   - Weights sit in HBM in MFMA operand order, k-step-major (see wfrag_offset): a wavefront
//     fetches a 32-row x 16-k tile with one contiguous 1 KiB load straight into registers, no LDS,
//     no transpose, and keeps three pipeline stages of them in flight.
//   - Activations are carried as bf16 PAIRS, x = hi + lo (two planes in operand order, written
//     that way by the producing kernel): a single bf16 rounding of every activation costs more
//     accuracy than the 2e-2 logit tolerance allows at 8B scale, so each weight tile is multiplied
//     with both planes.  All wavefronts of a workgroup need all of them: they go from L2 into a
//     ring of five LDS stage buffers with direct-to-LDS loads, four stages ahead.
//   - A workgroup is 8 wavefronts (two per SIMD), all alike: 2 column groups x 4 k-groups (4 x 2 when the
//     batch has several blocks of rows, 8 x 1 for the LM head; see the shapes below).  A stage is one k-step of 16 per k-group;
//     k-group g works on the g-th of them for the 64 columns (two 32-column
//     tiles) of its column group and all rows of the block (MT 32-row tiles), and the k-groups'
//     sums are exchanged through LDS at the end and added in a fixed order, after which every wavefront stores a
//     share of the outputs.  This shape follows from three
//     per-CU limits that all sit within a factor of two of the HBM time: one wavefront sustains
//     only about 4-5 bytes per clock from L2, so the activation stream (twice the weight bytes per
//     CU) has to be issued by all eight; ds_read_b128 runs at about 64 bytes per clock, so each
//     activation tile read from LDS has to feed four MFMAs; and the MFMAs themselves need two
//     wavefronts per SIMD to hide each other's waits.
//   - Vector-memory loads retire in order under one counter, and the compiler cannot see that the
//     two streams are independent (it drains the counter before any LDS read that might alias a
//     direct-to-LDS load).  Both kinds of loads are therefore issued from inline assembly in a
//     fixed order, and the waits are written by hand from that order.
//   - Split-K over blockIdx.y gives every CU work on the narrow projections; partial sums go to a
//     [split, T, N] fp32 buffer that the following row kernel reduces in a fixed order (no float
//     atomics: results are reproducible run to run).
//   - Weights may also be stored in 8 bits (FP8 E4M3, a scale per output row) or 4 bits (FP4 E2M1, a power-of-two
//     scale per row and 32 k): the same tiles at half or a quarter of the bytes, widened to bf16 in registers by
//     the hardware conversions; everything else is unchanged.
//   - The weight tile is the A operand, the activation tile the B operand, so a lane ends up with
//     groups of 4 consecutive output columns of one row: float4 stores, and gate/up pairs for
//     SwiGLU in-lane.
//
// fp32 path: plain LDS-tiled FMA kernel, used by fp32 models (correctness configuration).
#include "sled_internal.h"

#include <stdlib.h>
#include <string.h>
#include <algorithm>
#include <type_traits>

namespace {

constexpr int PLANES = 2;    // activation planes: hi, lo
constexpr int NW = 2;        // 32-column tiles per wavefront
constexpr int WAVES = 8;     // = k-groups x column groups of a workgroup shape
constexpr int DEPTH = 3;     // weight stages in flight beyond the one in use
constexpr int NBUF = DEPTH + 1;
constexpr int AHEAD = DEPTH + 1;  // activation stages in flight beyond the one being read
constexpr int NXB = AHEAD + 1;    // LDS ring
// Two workgroup shapes (KG k-groups = k-steps of 16 per stage, CG column groups of 64 columns):
//   narrow  KG 4, CG 2: 128 columns, 64 k per stage.  Most workgroups per projection: the shape for one block of
//           rows (up to 128), where the chip has to be filled by column blocks and K slices alone.
//   wide    KG 2, CG 4: 256 columns, 32 k per stage.  Per MFMA it fetches two thirds of the bytes (half the
//           activations, the same weights): the shape for several row blocks, where the workgroups are many
//           anyway and the L2 -> CU path, not HBM, is what the MFMAs wait for.
//   broad   KG 1, CG 8: 512 columns, 16 k per stage, no sums to exchange at the end.  Per MFMA it fetches half the
//           bytes of the narrow shape; only a matrix with enough columns to fill the chip without K slices can use
//           it (the LM head), and only with four row tiles (a stage's eight activation tiles go one to a wavefront).
constexpr int NARROW_KG = 4, NARROW_CG = 2, WIDE_KG = 2, WIDE_CG = 4, BROAD_KG = 1, BROAD_CG = 8;
constexpr int NARROW_COLS = NARROW_CG * NW * 32;

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float float16_t;
typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4_t;

// s_waitcnt vmcnt(N) tied to the registers the awaited loads write: the compiler sees the assembly
// loads as complete when issued, so the data dependence has to run through the wait.
template <int N>
__device__ __forceinline__ void wait_loads(u32x4_t& a, u32x4_t& b) {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N) : "memory");
}

// Eight 8-bit weights (FP8 E4M3, the OCP flavour gfx950 converts in hardware) -> a bf16 MFMA operand: one
// instruction per pair, exact (three mantissa bits fit bf16's seven).
__device__ __forceinline__ bf16x8_t cvt_w8(uint32_t lo, uint32_t hi) {
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_hw;
    const u32x4_t p = {__builtin_bit_cast(uint32_t, (bf16x2_hw)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, false)),
                       __builtin_bit_cast(uint32_t, (bf16x2_hw)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, true)),
                       __builtin_bit_cast(uint32_t, (bf16x2_hw)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, false)),
                       __builtin_bit_cast(uint32_t, (bf16x2_hw)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, true))};
    return __builtin_bit_cast(bf16x8_t, p);
}

// Eight 4-bit weights (FP4 E2M1, low nibble first) times a power-of-two block scale -> a bf16 MFMA operand; exact
__device__ __forceinline__ bf16x8_t cvt_w4(uint32_t codes, float scale) {
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_hw;
    const u32x4_t p = {__builtin_bit_cast(uint32_t, (bf16x2_hw)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 0)),
                       __builtin_bit_cast(uint32_t, (bf16x2_hw)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 1)),
                       __builtin_bit_cast(uint32_t, (bf16x2_hw)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 2)),
                       __builtin_bit_cast(uint32_t, (bf16x2_hw)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 3))};
    return __builtin_bit_cast(bf16x8_t, p);
}

// the same for a single register (never pass one register twice to the two-operand form: the second operand would
// be a copy taken while the load is still in flight)
template <int N>
__device__ __forceinline__ void wait_load(u32x4_t& a) {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(a) : "n"(N) : "memory");
}

typedef __attribute__((__vector_size__(2 * sizeof(unsigned)))) unsigned u32x2_t;
// ... and for the two registers of a 4-bit stage (codes and scales)
template <int N>
__device__ __forceinline__ void wait_load4(u32x2_t& a, uint32_t& b) {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N) : "memory");
}

// MT: 32-row tiles of activations per block.  WB: bits per weight.  8 (see w8_offset): the wavefront's two column
// tiles come with ONE load per stage, are widened to bf16 in registers, and the accumulators are multiplied by the
// columns' scales on the way out.  4 (see w4_offset): one 8-byte load per stage for the codes and one 2-byte load
// for the two rows' block scales, which the widening instruction applies.
template <int MT, int EPI, int KG, int CG, int WB>
__global__ __launch_bounds__(64 * WAVES) void gemm_bf16_kernel(const bf16_t* __restrict__ Xp, size_t x_plane,
                                                               const bf16_t* __restrict__ Wp,
                                                               const void* __restrict__ scale_v, int NT, int KS,
                                                               int n_col, int n_split, int n_zb,
                                                               int T, int T_pad, int N, float* __restrict__ out,
                                                               bf16_t* __restrict__ out_act, size_t act_plane,
                                                               int F_act) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int STAGE_TILES = PLANES * MT * KG;  // 1 KiB operand tiles per stage, ordered [plane][row tile][k-step]
    constexpr int MY_TILES = STAGE_TILES / WAVES;  // = MT: tiles of a stage this wavefront fetches
    constexpr bool W8 = WB == 8, W4 = WB == 4;
    static_assert(WB == 16 || W8 || W4, "16-, 8- or 4-bit weights");
    constexpr int NWL = WB == 16 ? NW : 1;         // weight loads per stage
    constexpr int NSL = W4 ? 1 : 0;                // block-scale loads per stage
    constexpr int PER_ITER = MY_TILES + NWL + NSL; // vector-memory instructions a wavefront issues per stage
    const float* scale = static_cast<const float*>(scale_v);
    constexpr unsigned STAGE_BYTES = STAGE_TILES * 1024;
    static_assert(KG * CG == WAVES, "a workgroup is eight wavefronts");
    static_assert(STAGE_TILES % WAVES == 0, "stage does not divide among the wavefronts");
    static_assert(PER_ITER * DEPTH < 64, "too many loads in flight for the counter");
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int cg = wv & (CG - 1), kgi = wv / CG;
    // Workgroup -> (column block bx, K slice by, row block bz).  Workgroups go to the eight XCDs round
    // robin by their linear index, and each XCD has its own L2.  The row blocks of one weight tile
    // stream the same weight bytes, so they are given consecutive slots of ONE XCD: they run side by
    // side there and all but the first find the weights in that L2 instead of fetching them from HBM
    // again.  Weight tile t = by * n_col + bx lives on XCD t % 8.
    int bx, by, bz;
    {
        const int w = blockIdx.x, xcd = w & 7, local = w >> 3;
        bz = local % n_zb;
        const int t = (local / n_zb) * 8 + xcd;
        if (t >= n_col * n_split) return;  // the grid is rounded up to whole rounds of eight tiles
        bx = t % n_col;
        by = t / n_col;
    }
    // K slice `by`: K in units of KG * NBUF k-steps (one trip of the stage loop), dealt out as evenly as whole units
    // allow -- the first `urem` slices hold one unit more (the host sees to n_split <= units)
    const int units = KS / (KG * NBUF), ubase = units / n_split, urem = units - ubase * n_split;
    const int ks_begin = (by * ubase + min(by, urem)) * (KG * NBUF);
    const int n_stage = (ubase + (by < urem ? 1 : 0)) * NBUF;  // a positive multiple of NBUF
    const int mt_base = bz * MT;            // first 32-row tile handled by this block

    // ---- activations: this wavefront's tiles of stage 0 and where they land in a stage buffer -----
    const int row_lim = (T + 7) & ~7;
    const bf16_t* xsrc[MY_TILES];
    unsigned xdst[MY_TILES];
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) void*)smem;  // LDS byte address of the ring
#pragma unroll
    for (int j = 0; j < MY_TILES; j++) {
        const int i = j * WAVES + wv;
        const int g = i % KG, pb = i / KG, pl = pb / MT, b = pb - pl * MT;
        // Lanes whose row lies past the last token (rounded up to whole 128-byte lines of 8 rows) re-read
        // the tile's first line instead: the fetch unit merges them into that line's request, so padding
        // rows cost no L2 traffic.  What lands in their LDS bytes only reaches their own output rows.
        // A block may reach past the last row tile (the wide shape always takes four): such a tile re-reads the
        // last one, and its results are not stored.
        const int mt = min(mt_base + b, T_pad / 32 - 1);
        const int row = mt * 32 + (lane & 31);
        const int src_lane = row < row_lim ? lane : (lane & 32) + (lane & 7);
        xsrc[j] = Xp + pl * x_plane + ((size_t)mt * KS + ks_begin + g) * 512 + src_lane * 8;
        xdst[j] = lds_base + i * 1024;
    }
    // one direct-to-LDS load moves a whole operand tile: lane l's 16 bytes land at m0 + 16*l
    auto x_issue_one = [&](int buf, int stage, int j) {
        const bf16_t* src = xsrc[j] + (size_t)stage * (KG * 512);
        const unsigned dst = __builtin_amdgcn_readfirstlane(xdst[j] + (unsigned)buf * STAGE_BYTES);
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(dst) : "memory");
    };
    auto x_issue = [&](int buf, int stage) {
#pragma unroll
        for (int j = 0; j < MY_TILES; j++) x_issue_one(buf, stage, j);
    };

    // ---- weights: NW tiles per stage, straight into registers ------------------------------------------
    const int nt0 = (bx * CG + cg) * NW;
    const int NTW = WB == 16 ? NT : NT / NW;  // blocks per k-step (an 8- or 4-bit block holds the wavefront's two tiles)
    constexpr int WBLK = W4 ? 256 : 512;      // size of a block and of a lane's share, in 2-byte units
    constexpr int WLANE = W4 ? 4 : 8;
    bool nt_ok[NW];
    const bf16_t* wsrc[NW];
#pragma unroll
    for (int a = 0; a < NW; a++) {
        nt_ok[a] = (nt0 + a) < NT;
        const int blk = WB == 16 ? nt0 + a : nt0 / NW;
        wsrc[a] = Wp + ((size_t)(ks_begin + kgi) * NTW + (nt_ok[a] ? blk : 0)) * WBLK + lane * WLANE;
    }
    // 4-bit weights: the scale bytes of this lane's row in both tiles; those of k-block kb lie kb * NTW * 64 bytes on
    const uint8_t* ssrc = static_cast<const uint8_t*>(scale_v);
    if (W4) ssrc += (size_t)(nt_ok[0] ? nt0 / NW : 0) * 64 + (lane & 31) * 2;
    u32x4_t wreg[NBUF][NWL];
    u32x2_t w4reg[NBUF];
    uint32_t sreg[NBUF];
    auto w_issue_one = [&](int buf, int stage, int a) {  // a: which of the stage's NWL + NSL weight-side loads
        const bf16_t* src = wsrc[a < NWL ? a : 0] + (size_t)stage * KG * NTW * WBLK;
        if (W4) {
            if (a == 0)
                asm volatile("global_load_dwordx2 %0, %1, off" : "=&v"(w4reg[buf]) : "v"(src) : "memory");
            else
                asm volatile("global_load_ushort %0, %1, off"
                             : "=&v"(sreg[buf])
                             : "v"(ssrc + (size_t)((ks_begin + kgi + stage * KG) >> 1) * NTW * 64)  // a k-block is two k-steps
                             : "memory");
        } else {
            asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(wreg[buf][a]) : "v"(src) : "memory");
        }
    };
    auto w_issue = [&](int buf, int stage) {
#pragma unroll
        for (int a = 0; a < NWL + NSL; a++) w_issue_one(buf, stage, a);
    };

    float16_t acc[NW][MT];
#pragma unroll
    for (int a = 0; a < NW; a++)
#pragma unroll
        for (int b = 0; b < MT; b++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[a][b][e] = 0.f;

    const bf16_t* xs = reinterpret_cast<const bf16_t*>(smem) + kgi * 512 + lane * 8;
    struct xfrag {
        bf16x8_t hi, lo;
    };
    auto read_x = [&](int xbuf, int b) {
        const bf16_t* xb = xs + (size_t)xbuf * (STAGE_BYTES / 2);
        xfrag f;
        f.hi = *reinterpret_cast<const bf16x8_t*>(xb + (size_t)b * (KG * 512));
        f.lo = *reinterpret_cast<const bf16x8_t*>(xb + (size_t)(MT + b) * (KG * 512));
        return f;
    };
    auto mfma4 = [&](int b, const xfrag& f, const bf16x8_t& w0, const bf16x8_t& w1) {
        acc[0][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w0, f.hi, acc[0][b], 0, 0, 0);
        acc[1][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1, f.hi, acc[1][b], 0, 0, 0);
        acc[0][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w0, f.lo, acc[0][b], 0, 0, 0);
        acc[1][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1, f.lo, acc[1][b], 0, 0, 0);
    };
    // One stage ("iteration" s): arithmetic of stage s, and the loads of later stages.
    //   - The iteration's PER_ITER loads (activations of stage s+AHEAD, then weights of stage
    //     s+DEPTH, always in that order) leave first, right after the wait.
    //   - LDS reads run one row tile ahead of the MFMAs that use them, and the first row tile of the
    //     next stage is read before the last MFMAs of this one.  `cur` holds row tile 0 of the stage
    //     on entry and row tile 0 of the next stage on exit.
    //   - The barrier before the last row tile says two things: this wavefront's share of stage s+1
    //     has landed (the wait at the top covers it), and its LDS reads of stage s are back, so that
    //     buffer may be refilled.
    // The wait at the top is for the weights of stage s and the activations of stage s+1, both issued
    // DEPTH iterations earlier; AFTER is the number of loads issued since.
    xfrag cur;
    auto stage = [&](auto after_c, int xbuf, auto wbuf_c, bool more, int x_stage, int x_buf, int w_stage) {
        constexpr int AFTER = decltype(after_c)::value, WBUF = decltype(wbuf_c)::value;
        bf16x8_t w0, w1;
        if (W4) {
            wait_load4<AFTER>(w4reg[WBUF], sreg[WBUF]);
            const uint32_t sb = sreg[WBUF];  // E8M0 bytes: 2^(e - 127) is the float with exponent field e
            w0 = cvt_w4(w4reg[WBUF][0], __uint_as_float((sb & 0xffu) << 23));
            w1 = cvt_w4(w4reg[WBUF][1], __uint_as_float((sb >> 8) << 23));
        } else if (W8) {
            wait_load<AFTER>(wreg[WBUF][0]);
            const u32x4_t r = wreg[WBUF][0];
            w0 = cvt_w8(r[0], r[1]);
            w1 = cvt_w8(r[2], r[3]);
        } else {
            wait_loads<AFTER>(wreg[WBUF][0], wreg[WBUF][NWL - 1]);
            w0 = __builtin_bit_cast(bf16x8_t, wreg[WBUF][0]);
            w1 = __builtin_bit_cast(bf16x8_t, wreg[WBUF][NWL - 1]);
        }
        auto issue = [&](int lo, int hi) {  // loads number lo .. hi-1 of this iteration
#pragma unroll
            for (int i = lo; i < hi; i++) {
                if (i < MY_TILES) {
                    if (x_stage >= 0) x_issue_one(x_buf, x_stage, i);
                } else {
                    if (w_stage >= 0) w_issue_one((WBUF + DEPTH) % NBUF, w_stage, i - MY_TILES);
                }
            }
        };
        issue(0, PER_ITER);
#pragma unroll
        for (int b = 0; b + 1 < MT; b++) {
            const xfrag nxt = read_x(xbuf, b + 1);
            __builtin_amdgcn_sched_barrier(0);
            mfma4(b, cur, w0, w1);
            __builtin_amdgcn_sched_barrier(0);
            cur = nxt;
        }
        __builtin_amdgcn_s_waitcnt(7 << 4 | 3 << 14 | 15);  // lgkmcnt(0) only
        __builtin_amdgcn_s_barrier();
        xfrag nxt = cur;
        if (more) nxt = read_x(xbuf == NXB - 1 ? 0 : xbuf + 1, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfma4(MT - 1, cur, w0, w1);
        __builtin_amdgcn_sched_barrier(0);
        cur = nxt;
    };
    using std::integral_constant;

    // prologue: activations of stages 0..DEPTH and weights of stages 0..DEPTH-1, in iteration order
    x_issue(0, 0);
#pragma unroll
    for (int u = 0; u < DEPTH; u++) {
        x_issue(u + 1, u + 1);
        w_issue(u, u);
    }
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(DEPTH * PER_ITER) : "memory");  // own tiles of stage 0
    __builtin_amdgcn_s_barrier();                                           // everybody's
    cur = read_x(0, 0);
    int xbuf = 0, fbuf = AHEAD;  // buffer being read; buffer the next activations go to
    int s0 = 0;
    auto advance = [&]() {
        xbuf = xbuf == NXB - 1 ? 0 : xbuf + 1;
        fbuf = fbuf == NXB - 1 ? 0 : fbuf + 1;
    };
    constexpr int STEADY = (DEPTH - 1) * PER_ITER;  // iterations s-DEPTH+1 .. s-1 have issued all their loads
    static_assert(DEPTH == 3 && NBUF == 4, "the trips below are written for three stages in flight");
    for (; s0 + NBUF < n_stage; s0 += NBUF) {
        // buffer fbuf held stage s-1: every reader passed the barrier of the previous iteration
        stage(integral_constant<int, STEADY>{}, xbuf, integral_constant<int, 0>{}, true, s0 + AHEAD, fbuf, s0 + DEPTH);
        advance();
        stage(integral_constant<int, STEADY>{}, xbuf, integral_constant<int, 1>{}, true, s0 + 1 + AHEAD, fbuf, s0 + 1 + DEPTH);
        advance();
        stage(integral_constant<int, STEADY>{}, xbuf, integral_constant<int, 2>{}, true, s0 + 2 + AHEAD, fbuf, s0 + 2 + DEPTH);
        advance();
        stage(integral_constant<int, STEADY>{}, xbuf, integral_constant<int, 3>{}, true, s0 + 3 + AHEAD, fbuf, s0 + 3 + DEPTH);
        advance();
    }
    // last trip: only the weights of the last stage are left to fetch (in its first iteration)
    stage(integral_constant<int, STEADY>{}, xbuf, integral_constant<int, 0>{}, true, -1, 0, s0 + DEPTH);
    advance();
    stage(integral_constant<int, PER_ITER + NWL + NSL>{}, xbuf, integral_constant<int, 1>{}, true, -1, 0, -1);
    advance();
    stage(integral_constant<int, NWL + NSL>{}, xbuf, integral_constant<int, 2>{}, true, -1, 0, -1);
    advance();
    stage(integral_constant<int, 0>{}, xbuf, integral_constant<int, 3>{}, false, -1, 0, -1);
    __syncthreads();  // every stage has been consumed and no load is in flight: the ring is free

    // ---- add the k-groups' sums through LDS ------------------------------------------------------------------------
    // A lane holds, per (column tile a, row tile b), four groups q of four consecutive columns: 4 * MT units
    // u = 4 * b + q per column tile.  The KG wavefronts that share a column group divide the units among themselves
    // in runs (k-group g owns units g * UPW .. (g + 1) * UPW - 1, i.e. whole row tiles when MT is a multiple of KG, so
    // that the stores of one wavefront fill whole 128-byte lines of an output row): each sends the units it does not
    // own to their owners and adds what it receives to its own, always in ascending k-group order.  Afterwards all
    // eight wavefronts hold a disjoint share of the block's outputs and all of them run the epilogue.
    // With two k-groups (the wide shape) k-group 0 owns everything instead and k-group 1 is done after sending: measured
    // 2 % faster there than sharing the epilogue, while with four k-groups four owners beat two (by 2 %) and one (by 20 %).
    constexpr int NOWN = KG == 2 ? 1 : KG;  // owning k-groups (0 .. NOWN-1)
    constexpr int UPW = 4 * MT / NOWN;               // units per owning wavefront and column tile
    auto owner = [](int b2, int q) { return (4 * b2 + q) / UPW; };
    // both column tiles in one pass where the parcels of both fit into the CU's 160 KiB, else one tile per pass
    constexpr int PARCELS_PER_TILE = CG * NOWN * (KG - 1) * UPW;  // KiB
    constexpr int PASSES = PARCELS_PER_TILE * NW <= 160 ? 1 : NW, TILES_PER_PASS = NW / PASSES;
    if (KG > 1) {
        float4_t* red = reinterpret_cast<float4_t*>(smem);
        // parcel (destination k-group, source k-group, unit, column tile within the pass): 64 lanes x 16 bytes
        auto parcel = [&](int dest, int src, int u, int ap) {
            // the destination has no slot of its own; src == dest is never accessed and maps to slot 0 to stay in range
            const int s2 = src < dest ? src : (src > dest ? src - 1 : 0);
            const int slot = ((cg * NOWN + dest) * (KG - 1) + s2) * UPW + (u - dest * UPW);
            return red + ((size_t)(slot * TILES_PER_PASS + ap)) * 64 + lane;
        };
#pragma unroll
        for (int pass = 0; pass < PASSES; pass++) {
#pragma unroll
            for (int ap = 0; ap < TILES_PER_PASS; ap++) {
                const int a = pass * TILES_PER_PASS + ap;
#pragma unroll
                for (int b2 = 0; b2 < MT; b2++)
#pragma unroll
                    for (int q = 0; q < 4; q++)
                        if (owner(b2, q) != kgi)
                            *parcel(owner(b2, q), kgi, 4 * b2 + q, ap) =
                                float4_t{acc[a][b2][4 * q], acc[a][b2][4 * q + 1], acc[a][b2][4 * q + 2], acc[a][b2][4 * q + 3]};
            }
            __syncthreads();
#pragma unroll
            for (int ap = 0; ap < TILES_PER_PASS; ap++) {
                const int a = pass * TILES_PER_PASS + ap;
#pragma unroll
                for (int b2 = 0; b2 < MT; b2++)
#pragma unroll
                    for (int q = 0; q < 4; q++)
                        if (owner(b2, q) == kgi) {
                            const float4_t own = {acc[a][b2][4 * q], acc[a][b2][4 * q + 1], acc[a][b2][4 * q + 2], acc[a][b2][4 * q + 3]};
                            float4_t v = kgi == 0 ? own : *parcel(kgi, 0, 4 * b2 + q, ap);
#pragma unroll
                            for (int src = 1; src < KG; src++) v += kgi == src ? own : *parcel(kgi, src, 4 * b2 + q, ap);
#pragma unroll
                            for (int i = 0; i < 4; i++) acc[a][b2][4 * q + i] = v[i];
                        }
            }
            if (pass + 1 < PASSES) __syncthreads();  // the parcels have been read: the next pass may overwrite them
        }
        if (kgi >= NOWN) return;
    }

    // epilogue: lane holds row (token) mt*32 + lane%32 and, in registers 4q .. 4q+3, the columns
    // nt*32 + 8q + (lane/32)*4 + 0..3; a wavefront stores the units it owns
#pragma unroll
    for (int a = 0; a < NW; a++) {
        if (!nt_ok[a]) continue;
        float4_t sc[4];
        if (W8) {  // 8-bit weights: the columns' scales
#pragma unroll
            for (int q = 0; q < 4; q++) sc[q] = *reinterpret_cast<const float4_t*>(scale + (nt0 + a) * 32 + q * 8 + (lane >> 5) * 4);
        }
#pragma unroll
        for (int b = 0; b < MT; b++) {
            const int tok = (mt_base + b) * 32 + (lane & 31);
#pragma unroll
            for (int q = 0; q < 4; q++) {
                if (owner(b, q) != kgi) continue;
                const int n = (nt0 + a) * 32 + q * 8 + (lane >> 5) * 4;
                float4_t v = {acc[a][b][4 * q], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]};
                if (W8) v *= sc[q];
                if (EPI == SLED_EPI_PARTIAL) {
                    if (tok < T) *reinterpret_cast<float4_t*>(out + ((size_t)by * T_pad + tok) * N + n) = v;  // padding rows are never read
                } else if (EPI == SLED_EPI_STORE) {
                    if (tok < T) *reinterpret_cast<float4_t*>(out + (size_t)tok * N + n) = v;
                } else {  // SwiGLU: columns are (gate f, up f, gate f+1, up f+1)
                    if (tok < T) {  // padding rows: what a consumer reads there only reaches its own padding rows
                        const int f = n >> 1;
                        const float a0 = v[0] / (1.f + __expf(-v[0])) * v[1];
                        const float a1 = v[2] / (1.f + __expf(-v[2])) * v[3];
                        const bf16_t h0 = f32_to_bf16(a0), h1 = f32_to_bf16(a1);
                        const bf16_t l0 = f32_to_bf16(a0 - bf16_to_f32(h0)), l1 = f32_to_bf16(a1 - bf16_to_f32(h1));
                        const size_t o = frag_offset(tok, f, F_act);
                        *reinterpret_cast<uint32_t*>(out_act + o) = (uint32_t)h0 | ((uint32_t)h1 << 16);
                        *reinterpret_cast<uint32_t*>(out_act + act_plane + o) = (uint32_t)l0 | ((uint32_t)l1 << 16);
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------ fp32
// out[t][n] = sum_k X[t][k] W[n][k]; block = 16 tokens x 64 columns, 256 threads, each 4 tokens x 1 column
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ X, const float* __restrict__ W, int T,
                                                       int N, int K, float* __restrict__ out) {
    __shared__ float xs[16][33];
    __shared__ float ws[64][33];
    const int tid = threadIdx.x;
    const int n0 = blockIdx.x * 64, t0 = blockIdx.y * 16;
    const int tx = tid & 63, ty = tid >> 6;  // column, token group
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < K; k0 += 32) {
        for (int e = tid; e < 16 * 32; e += 256) {
            int r = e >> 5, c = e & 31;
            xs[r][c] = (t0 + r < T && k0 + c < K) ? X[(size_t)(t0 + r) * K + k0 + c] : 0.f;
        }
        for (int e = tid; e < 64 * 32; e += 256) {
            int r = e >> 5, c = e & 31;
            ws[r][c] = (n0 + r < N && k0 + c < K) ? W[(size_t)(n0 + r) * K + k0 + c] : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int c = 0; c < 32; c++) {
            float w = ws[tx][c];
#pragma unroll
            for (int i = 0; i < 4; i++) acc[i] = fmaf(xs[ty * 4 + i][c], w, acc[i]);
        }
        __syncthreads();
    }
    const int n = n0 + tx;
    if (n < N)
        for (int i = 0; i < 4; i++) {
            int t = t0 + ty * 4 + i;
            if (t < T) out[(size_t)t * N + n] = acc[i];
        }
}

struct gemm_args {
    dim3 grid;
    size_t lds;
    hipStream_t st;
    const bf16_t* X;
    size_t x_plane;
    const bf16_t* W;
    const void* scale;
    int wbits;
    int NT, KS, n_col, n_split, n_zb, T, T_pad, N;
    float* out;
    bf16_t* out_act;
    size_t act_plane;
    int F_act;
};

template <int MT, int EPI, int KG, int CG, int WB>
int launch_one(const gemm_args& a) {
    // more than 64 KiB of dynamic LDS has to be allowed once per kernel
    static bool allowed = false;
    auto kern = gemm_bf16_kernel<MT, EPI, KG, CG, WB>;
    if (!allowed) {
        SLED_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)a.lds));
        allowed = true;
    }
    hipLaunchKernelGGL(kern, a.grid, dim3(64 * WAVES), a.lds, a.st, a.X, a.x_plane, a.W, a.scale, a.NT, a.KS, a.n_col,
                       a.n_split, a.n_zb, a.T, a.T_pad, a.N, a.out, a.out_act, a.act_plane, a.F_act);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

template <int MT, int KG, int CG, int WB>
int launch_epi_wb(int epi, const gemm_args& a) {
    switch (epi) {
        case SLED_EPI_PARTIAL: return launch_one<MT, SLED_EPI_PARTIAL, KG, CG, WB>(a);
        case SLED_EPI_SWIGLU: return launch_one<MT, SLED_EPI_SWIGLU, KG, CG, WB>(a);
        default: return launch_one<MT, SLED_EPI_STORE, KG, CG, WB>(a);
    }
}

template <int MT, int KG, int CG>
int launch_epi(int epi, const gemm_args& a) {
    switch (a.wbits) {
        case 8: return launch_epi_wb<MT, KG, CG, 8>(epi, a);
        case 4: return launch_epi_wb<MT, KG, CG, 4>(epi, a);
        default: return launch_epi_wb<MT, KG, CG, 16>(epi, a);
    }
}

}  // namespace

// Number of K slices for a projection of N columns over K.  More slices mean more workgroups (the
// chip wants at least one per CU) but more partial sums to reduce.  Each slice must hold a multiple
// of 4 stages of 64 k.
static sled_gemm_plan plan_one_block(int N, int K, bool needs_full_k);
static sled_gemm_plan plan_for_rows(sled_gemm_plan base, int N, int K, int T_pad);

sled_gemm_plan sled_gemm_make_plan(const sled_model* m, int N, int K, bool needs_full_k) {
    if (m->s.dtype != SLED_BF16) return sled_gemm_plan{1, 1};
    return plan_one_block(N, K, needs_full_k);
}

static sled_gemm_plan plan_one_block(int N, int K, bool needs_full_k) {
    sled_gemm_plan p{1, 1};
    auto legal = [&](int sp) { return sp >= 1 && (K / 16) % (sp * NARROW_KG * NBUF) == 0; };
    const int n_wg = (N + NARROW_COLS - 1) / NARROW_COLS;
    if (!needs_full_k)
        while (n_wg * p.split < 160 && legal(p.split * 2)) p.split *= 2;
    // a step with several blocks of rows may pick another number of slices, up to twice as many
    p.cap = needs_full_k || p.split == 1 ? p.split : std::min(2 * p.split, K / 16 / (NARROW_KG * NBUF));
    return p;
}

// With more than one block of rows (the wide shape) the workgroups of a projection are column blocks x row blocks x
// K slices, and what counts is how many rounds of 256 they make: 288 workgroups take as long as 512.  Fewer K slices
// also mean fewer partial sums to write and to read back.  Estimated time of a launch, in microseconds: rounds x
// (fixed part + stages per workgroup x time per stage) + bytes of partial sums written and read / rate.
sled_gemm_plan sled_gemm_plan_rows(const sled_model* m, sled_gemm_plan base, int N, int K, int T_pad) {
    if (m->s.dtype != SLED_BF16 || m->batch_invariant) return base;
    return plan_for_rows(base, N, K, T_pad);
}

static sled_gemm_plan plan_for_rows(sled_gemm_plan base, int N, int K, int T_pad) {
    if (base.split <= 1 || T_pad / 32 <= 4) return base;
    constexpr double FIXED_US = 9.0, STAGE_US = 0.8, PARTIAL_BYTES_PER_US = 4.0e6;
    const int n_col = (N / 32 + WIDE_CG * NW - 1) / (WIDE_CG * NW), zb = (T_pad / 32 + 3) / 4;
    const int units = K / 16 / (WIDE_KG * NBUF);   // trips of the stage loop in all of K
    sled_gemm_plan best = base;
    double best_t = -1.0;
    for (int sp = 1; sp <= base.cap && sp <= units; sp++) {
        const int64_t wgs = (int64_t)n_col * zb * sp;
        const int stages = (units + sp - 1) / sp * NBUF;   // of the longest slice
        const double t = (double)((wgs + 255) / 256) * (FIXED_US + stages * STAGE_US) + 2.0 * sp * (double)T_pad * N * 4.0 / PARTIAL_BYTES_PER_US;
        if (best_t < 0 || t < best_t) {
            best_t = t;
            best.split = sp;
        }
    }
    return best;
}

extern "C" int sled_projection_slices(int n_out, int n_in, int T, int* slices /*host out*/, int* max_slices /*host out*/) {
    if (!slices || !max_slices || n_out < 32 || n_in < 16 * NARROW_KG * NBUF || n_out % 32 || n_in % (16 * NARROW_KG * NBUF) || T < 1)
        SLED_FAIL(SLED_EINVAL, "sled_projection_slices: bad argument");
    const sled_gemm_plan base = plan_one_block(n_out, n_in, false);
    *slices = plan_for_rows(base, n_out, n_in, (T + 31) / 32 * 32).split;
    *max_slices = base.cap;
    return SLED_OK;
}

int sled_launch_gemm(const sled_model* m, const void* X, size_t x_plane, const void* W, const void* scale, int T, int T_pad,
                     int N, int K, int epilogue, sled_gemm_plan plan, float* out_f32, void* out_act, size_t act_plane,
                     int F_act, hipStream_t st) {
    if (m->s.dtype == SLED_BF16) {
        const int NT = N / 32, KS = K / 16;
        if (N % 32 || K % 16 || T_pad % 32 || plan.split < 1 || KS % (NARROW_KG * NBUF) || plan.split > KS / (NARROW_KG * NBUF))
            SLED_FAIL(SLED_EINVAL, "gemm: unsupported shape N=%d K=%d T_pad=%d split=%d", N, K, T_pad, plan.split);
        const int mt_total = T_pad / 32;
        // rows are processed in blocks of at most 4 tiles (128 rows): one block -> narrow shape with exactly its
        // tiles; several -> wide shape, four tiles each (the last block may reach past the end)
        // (a batch-invariant model keeps the narrow shape at every size: the two shapes add the k-steps up in
        // different groupings, so a row's sums would depend on whether its batch has more than 128 rows)
        const bool wide = mt_total > 4 && !m->batch_invariant;
        const int zb = (mt_total + 3) / 4;
        const int MT = wide ? 4 : (mt_total + zb - 1) / zb;
        // one block of four row tiles, no K slices, and column blocks of 512 that fill at least three quarters of the CUs
        const bool broad = !wide && MT == 4 && plan.split == 1 && !m->batch_invariant && (NT + BROAD_CG * NW - 1) / (BROAD_CG * NW) >= 192;
        const int KG = wide ? WIDE_KG : broad ? BROAD_KG : NARROW_KG, CG = wide ? WIDE_CG : broad ? BROAD_CG : NARROW_CG;
        gemm_args a;
        a.n_col = (NT + CG * NW - 1) / (CG * NW);
        a.n_split = plan.split;
        a.n_zb = zb;
        a.grid = dim3((a.n_col * a.n_split + 7) / 8 * 8 * a.n_zb, 1, 1);
        // the ring of activation stages; afterwards the same memory holds the parcels the k-groups exchange
        // (every wavefront sends (KG - 1) / KG of its MT * 4 groups of 1 KiB per column tile)
        const size_t parcels = (size_t)WAVES * (KG - 1) * (4 * MT / KG);  // KiB per column tile; both tiles at once if they fit
        a.lds = std::max((size_t)NXB * PLANES * MT * KG * 1024, (parcels * NW <= 160 ? parcels * NW : parcels) * 1024);
        a.st = st;
        a.X = static_cast<const bf16_t*>(X);
        a.x_plane = x_plane;
        a.W = static_cast<const bf16_t*>(W);
        a.wbits = m->wbits;
        a.scale = m->wbits != 16 ? scale : nullptr;
        if (m->wbits != 16 && (!scale || N % 64 || K % 32))
            SLED_FAIL(SLED_EINVAL, "gemm: %d-bit weights need scales, N (%d) a multiple of 64 and K (%d) of 32", m->wbits, N, K);
        a.NT = NT;
        a.KS = KS;
        a.T = T;
        a.T_pad = T_pad;
        a.N = N;
        a.out = out_f32;
        a.out_act = static_cast<bf16_t*>(out_act);
        a.act_plane = act_plane;
        a.F_act = F_act;
        if (wide) return launch_epi<4, WIDE_KG, WIDE_CG>(epilogue, a);
        if (broad) return launch_epi<4, BROAD_KG, BROAD_CG>(epilogue, a);
        switch (MT) {
            case 1: return launch_epi<1, NARROW_KG, NARROW_CG>(epilogue, a);
            case 2: return launch_epi<2, NARROW_KG, NARROW_CG>(epilogue, a);
            case 3: return launch_epi<3, NARROW_KG, NARROW_CG>(epilogue, a);
            default: return launch_epi<4, NARROW_KG, NARROW_CG>(epilogue, a);
        }
    }
    // fp32: no split, plain store (partial buffer with one slice has the same layout)
    dim3 grid((N + 63) / 64, (T + 15) / 16);
    hipLaunchKernelGGL(gemm_f32_kernel<0>, grid, dim3(256), 0, st, static_cast<const float*>(X),
                       static_cast<const float*>(W), T, N, K, out_f32);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}
