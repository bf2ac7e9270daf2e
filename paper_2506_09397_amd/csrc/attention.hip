// Ragged speculative-verify attention over the paged K/V cache.
//
// Request i contributes n_i = k_i + 1 query rows at positions L_i .. L_i + k_i.  Row j attends to
// every context key and to the new keys up to itself: a causal mask that only matters on the last
// one or two pages.  All G query heads that share a kv head and all n_i rows of the request are
// stacked into one tile of G * n_i "query rows", so each K/V byte is fetched from HBM once per
// step and reused G * n_i times (this is the whole arithmetic intensity the step has).
//
// bf16 kernel, per work item (request, kv head, run of pages):
//   S^T[token, qrow] = K_page * Q^T      v_mfma_f32_16x16x32_bf16, K page tile as the A operand; q is a
//                                        bf16 pair (hi + lo, two MFMAs), its tiles sit in LDS
//   online softmax per qrow              (a lane owns one qrow: reductions over 4 registers and
//                                         2 cross-lane steps); the running maximum is rounded up
//                                         to a whole number of log2 units, so the numerators
//                                         p = 2^(s - M) are rounded to bf16 the same way whatever
//                                         the page order or the split of the keys over wavefronts
//   O^T[d, qrow]    += V_page^T * P^T    v_mfma_f32_16x16x16_bf16; the S^T accumulator registers
//                                        are, in place, the P^T operand (p too is a bf16 pair)
// A page (16 tokens x 128 dims of one kv head) is stored in the pool in operand order, K for the
// first product and V for the second, so a page moves with 4 + 4 contiguous 1 KiB direct-to-LDS loads.
// A workgroup is NPG page groups of QT consumer wavefronts and one producer wavefront: the producer
// streams every NPG-th page of the work item through the group's ring of three LDS page buffers (two
// pages in flight), and each consumer computes one tile of 16 query rows against the page.  One
// barrier per round keeps the groups in step.  At the end the groups' (max, sum, O) states are folded
// through LDS.  When a (request, kv head) is split over several work items, each stores its state and
// the last one to arrive (a device-scope counter) merges them in a fixed order; either way the
// output is written in the operand order of the following projection, as a bf16 pair.
// FUSED (a verification step: every block is a request of its own): the kernel starts from the K-slice partial sums
// of the QKV projection.  Each consumer wavefront adds up, rotates and splits into a bf16 pair the q rows of its own
// tile; the consumers together do the same for the request's new k and v rows of this kv head and write them into
// the cache pages (the work item that holds a row's page does), while the producers already stream the context
// pages, which depend on none of this.  Only the pages that hold new rows wait for those stores.
//
// fp32 kernel (fp32 models): one wavefront per (row, query head), lanes over keys.
#include "sled_internal.h"

namespace {

constexpr float NEG_BIG = -1.0e30f;

// Wavefronts of a workgroup: NPG page groups x (QT consumers + 1 producer).  Page group p takes the
// pages page0 + p, + NPG, ... of the work item; its consumer qt owns the 16 query rows of tile qt, its
// producer does nothing but move the group's pages into LDS.  Several wavefronts per SIMD hide each
// other's dependent chains (S^T -> softmax -> O^T); the producer is separate because a wavefront
// issues in order and a direct-to-LDS load can hold the issue slot for a couple of hundred clocks.
__host__ __device__ constexpr int attn_groups(int QT) { return QT <= 3 ? 4 : (QT == 4 ? 3 : 2); }
constexpr int ATTN_RING = 3;  // page buffers per page group: the one being read and two in flight

// floats of one parked state in LDS: O tile [8][64 lanes][4] + max[16] + sum[16]
constexpr int ATTN_PARK_F = 8 * 64 * 4 + 32;

template <int QT, bool FUSED>
__global__ __launch_bounds__(64 * (QT + 1) * attn_groups(QT)) void attn_bf16_kernel(
    sled_step_meta meta, const int32_t* __restrict__ len_dev, const bf16_t* __restrict__ Q, size_t q_plane,
    const float* __restrict__ qkv_partial, int n_split, int T_pad, const float2* __restrict__ cs,
    const int32_t* __restrict__ kvslot, const int32_t* __restrict__ plan, bf16_t* k_pool, bf16_t* v_pool, int64_t n_pages,
    int layer, int Hq, int Hkv,
    float scale_log2, float* __restrict__ part_o, float* __restrict__ part_ml, int32_t* __restrict__ arrive,
    bf16_t* __restrict__ X, size_t x_plane) {
    constexpr int D = 128, NPG = attn_groups(QT), RING = ATTN_RING;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ int sh_last;

    const int w = blockIdx.x;
    // the work item's record, written once per step by attn_plan_kernel: one look-up instead of a chain of four
    const int32_t* rec = plan + 12 * w;
    const int b = rec[0], g = rec[1];
    const int page0 = rec[2], npg = rec[3];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: page ids are then fetched by scalar loads
    const bool producer = wv >= NPG * QT;
    const int pgid = producer ? wv - NPG * QT : wv / QT, qt = producer ? 0 : wv - pgid * QT;
    const int G = Hq / Hkv;
    const int L = rec[4];  // everything before the block's first row is context
    const int n = rec[5];
    const int rows = G * n;
    const int row0 = rec[6];
    const int n_valid_pages = (L + n + 15) >> 4;
    const int page_end = min(page0 + npg, n_valid_pages);
    const int32_t* pages = meta.pages + rec[7];
    const int lq = lane & 15, lg = lane >> 4;

    // Q operand of this wavefront's tile, both planes of the bf16 pair, straight into registers:
    // qrow r = qt*16 + l%16 -> (query position j = r / G, head g*G + r % G); element k = ks*32 + (l/16)*8 ..+8
    const int r_mine = qt * 16 + lq;
    const int jrow = r_mine / G;
    bf16x8_t qf[2][4];
#pragma unroll
    for (int pl = 0; pl < 2; pl++)
#pragma unroll
        for (int ks = 0; ks < 4; ks++) qf[pl][ks] = __builtin_bit_cast(bf16x8_t, make_uint4(0u, 0u, 0u, 0u));
    if (!FUSED) {
        const int hh = r_mine - jrow * G;
#pragma unroll
        for (int pl = 0; pl < 2; pl++)
#pragma unroll
            for (int ks = 0; ks < 4; ks++) {
                uint4 val = make_uint4(0u, 0u, 0u, 0u);
                if (!producer && r_mine < rows)
                    val = *reinterpret_cast<const uint4*>(Q + pl * q_plane + ((size_t)(row0 + jrow) * Hq + g * G + hh) * D +
                                                          ks * 32 + lg * 8);
                qf[pl][ks] = __builtin_bit_cast(bf16x8_t, val);
            }
    } else if (!producer) {
        // Items: QT*16 rows x 16 quads of q (a quad = four neighbouring rotary pairs of one head: dims i..i+3 and
        // i+64..i+67), then n x 16 quads of k, then n x 32 groups of four v values.  Lane `me` of the consumers takes
        // items me, me + nc, ...; all loads of up to two items are in flight together, so the prologue costs one
        // round trip to the partial sums, not one per K slice.
        const int n_qkv = (Hq + 2 * Hkv) * D;
        const size_t sstride = (size_t)T_pad * n_qkv;   // one K slice of the projection
        const int nc = NPG * QT * 64, me = wv * 64 + lane;
        const int NQ = QT * 16 * 16, NK = n * 16, NV = n * 32;
        bf16_t* qtile = reinterpret_cast<bf16_t*>(smem) + (size_t)NPG * RING * 4096;   // behind the page rings
        for (int it0 = me; it0 < NQ + NK + NV; it0 += 2 * nc) {
            int kind[2];          // 0 q, 1 k, 2 v, -1 nothing to fetch
            int jr[2], ci[2];     // row (q: query row of the tile set; k, v: row of the request), quad / group index
            const float* src[2];  // first element of the item in K slice 0 (second quad of a rotary item 64 further)
            float4 acc[2][2];
#pragma unroll
            for (int u = 0; u < 2; u++) {
                const int it = it0 + u * nc;
                kind[u] = -1;
                jr[u] = ci[u] = 0;
                src[u] = qkv_partial;
                acc[u][0] = acc[u][1] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (it < NQ) {
                    jr[u] = it >> 4;
                    ci[u] = it & 15;
                    if (jr[u] < rows) {
                        const int j = jr[u] / G, hh = jr[u] - j * G;
                        kind[u] = 0;
                        src[u] = qkv_partial + (size_t)(row0 + j) * n_qkv + (g * G + hh) * D + 4 * ci[u];
                    }
                } else if (it < NQ + NK + NV) {
                    const bool isk = it < NQ + NK;
                    const int e = isk ? it - NQ : it - NQ - NK;
                    jr[u] = isk ? e >> 4 : e >> 5;
                    ci[u] = isk ? e & 15 : e & 31;
                    const int lp = (L + jr[u]) >> 4;
                    if (lp >= page0 && lp < page_end) {   // the row's page belongs to this work item
                        kind[u] = isk ? 1 : 2;
                        src[u] = qkv_partial + (size_t)(row0 + jr[u]) * n_qkv + (Hq + (isk ? 0 : Hkv) + g) * D + 4 * ci[u];
                    }
                }
            }
            for (int sp0 = 0; sp0 < n_split; sp0 += 4) {   // K slices in ascending order, four at a time
                float4 v[2][4][2];
#pragma unroll
                for (int u = 0; u < 2; u++)
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const bool on = kind[u] >= 0 && sp0 + q < n_split;
                        const float* ptr = src[u] + (size_t)(sp0 + q) * sstride;
                        v[u][q][0] = on ? *reinterpret_cast<const float4*>(ptr) : make_float4(0.f, 0.f, 0.f, 0.f);
                        v[u][q][1] = (on && kind[u] < 2) ? *reinterpret_cast<const float4*>(ptr + D / 2) : make_float4(0.f, 0.f, 0.f, 0.f);
                    }
#pragma unroll
                for (int u = 0; u < 2; u++)
#pragma unroll
                    for (int q = 0; q < 4; q++)
#pragma unroll
                        for (int h2 = 0; h2 < 2; h2++) {
                            acc[u][h2].x += v[u][q][h2].x;
                            acc[u][h2].y += v[u][q][h2].y;
                            acc[u][h2].z += v[u][q][h2].z;
                            acc[u][h2].w += v[u][q][h2].w;
                        }
            }
#pragma unroll
            for (int u = 0; u < 2; u++) {
                const int it = it0 + u * nc;
                if (it >= NQ + NK + NV) continue;
                const float x1[4] = {acc[u][0].x, acc[u][0].y, acc[u][0].z, acc[u][0].w};
                const float x2[4] = {acc[u][1].x, acc[u][1].y, acc[u][1].z, acc[u][1].w};
                if (it < NQ) {
                    // q quad -> the tile's operand image in LDS: row r = qt'*16 + lq', dim d -> [plane][d/32][lane (d%32/8)*16 + lq'][d%8]
                    uint32_t h1[2] = {0u, 0u}, l1[2] = {0u, 0u}, h2[2] = {0u, 0u}, l2[2] = {0u, 0u};
                    if (kind[u] == 0) {
                        const int j = jr[u] / G;
                        const float4 c01 = *reinterpret_cast<const float4*>(cs + (size_t)(row0 + j) * (D / 2) + 4 * ci[u]);
                        const float4 c23 = *reinterpret_cast<const float4*>(cs + (size_t)(row0 + j) * (D / 2) + 4 * ci[u] + 2);
                        const float cc[4] = {c01.x, c01.z, c23.x, c23.z}, ss[4] = {c01.y, c01.w, c23.y, c23.w};
                        float y1[4], y2[4];
#pragma unroll
                        for (int e = 0; e < 4; e++) rope_pair(x1[e], x2[e], cc[e], ss[e], y1[e], y2[e]);
#pragma unroll
                        for (int e2 = 0; e2 < 2; e2++) {
                            const bf16_t a0 = f32_to_bf16(y1[2 * e2]), a1 = f32_to_bf16(y1[2 * e2 + 1]);
                            const bf16_t b0 = f32_to_bf16(y2[2 * e2]), b1 = f32_to_bf16(y2[2 * e2 + 1]);
                            h1[e2] = (uint32_t)a0 | ((uint32_t)a1 << 16);
                            h2[e2] = (uint32_t)b0 | ((uint32_t)b1 << 16);
                            l1[e2] = (uint32_t)f32_to_bf16(y1[2 * e2] - bf16_to_f32(a0)) | ((uint32_t)f32_to_bf16(y1[2 * e2 + 1] - bf16_to_f32(a1)) << 16);
                            l2[e2] = (uint32_t)f32_to_bf16(y2[2 * e2] - bf16_to_f32(b0)) | ((uint32_t)f32_to_bf16(y2[2 * e2 + 1] - bf16_to_f32(b1)) << 16);
                        }
                    }
                    const int d = 4 * ci[u];   // < 64
                    const int tq = jr[u] >> 4, ldst = (((d & 31) >> 3) << 4) + (jr[u] & 15), ks = d >> 5;
                    bf16_t* base = qtile + (size_t)tq * 4096 + (size_t)ldst * 8 + (d & 7);
                    *reinterpret_cast<uint2*>(base + (0 * 4 + ks) * 512) = make_uint2(h1[0], h1[1]);
                    *reinterpret_cast<uint2*>(base + (1 * 4 + ks) * 512) = make_uint2(l1[0], l1[1]);
                    *reinterpret_cast<uint2*>(base + (0 * 4 + ks + 2) * 512) = make_uint2(h2[0], h2[1]);
                    *reinterpret_cast<uint2*>(base + (1 * 4 + ks + 2) * 512) = make_uint2(l2[0], l2[1]);
                } else if (kind[u] == 1) {
                    const int t = row0 + jr[u], i = 4 * ci[u];
                    const float4 c01 = *reinterpret_cast<const float4*>(cs + (size_t)t * (D / 2) + i);
                    const float4 c23 = *reinterpret_cast<const float4*>(cs + (size_t)t * (D / 2) + i + 2);
                    const float cc[4] = {c01.x, c01.z, c23.x, c23.z}, ss[4] = {c01.y, c01.w, c23.y, c23.w};
                    float y1[4], y2[4];
#pragma unroll
                    for (int e = 0; e < 4; e++) rope_pair(x1[e], x2[e], cc[e], ss[e], y1[e], y2[e]);
                    const int ps = kvslot[t];
                    bf16_t* kp = k_pool + (((size_t)layer * n_pages + (ps >> 4)) * Hkv + g) * (16 * D);
                    // four neighbouring dims share an 8-byte piece of the page's operand order
                    *reinterpret_cast<uint2*>(kp + kpage_offset(ps & 15, i)) =
                        make_uint2((uint32_t)f32_to_bf16(y1[0]) | ((uint32_t)f32_to_bf16(y1[1]) << 16),
                                   (uint32_t)f32_to_bf16(y1[2]) | ((uint32_t)f32_to_bf16(y1[3]) << 16));
                    *reinterpret_cast<uint2*>(kp + kpage_offset(ps & 15, i + D / 2)) =
                        make_uint2((uint32_t)f32_to_bf16(y2[0]) | ((uint32_t)f32_to_bf16(y2[1]) << 16),
                                   (uint32_t)f32_to_bf16(y2[2]) | ((uint32_t)f32_to_bf16(y2[3]) << 16));
                } else if (kind[u] == 2) {
                    const int t = row0 + jr[u], dd = 4 * ci[u];
                    const int ps = kvslot[t];
                    bf16_t* vp = v_pool + (((size_t)layer * n_pages + (ps >> 4)) * Hkv + g) * (16 * D);
#pragma unroll
                    for (int e = 0; e < 4; e++) vp[vpage_offset(ps & 15, dd + e)] = f32_to_bf16(x1[e]);
                }
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the hand-counted waits below start from an empty queue

    // the tile count follows the longest request the model allows; a request with fewer query rows
    // leaves the upper tiles' wavefronts without work (they only keep the barriers company)
    const bool active = qt * 16 < rows;
    float m = NEG_BIG, lsum = 0.f;
    float4_t o[8];
#pragma unroll
    for (int dt = 0; dt < 8; dt++) o[dt] = float4_t{0.f, 0.f, 0.f, 0.f};

    // K/V pages go from HBM straight into the page group's LDS ring (RING pages of 8 KiB) with
    // direct-to-LDS loads: 4 + 4 loads of 1 KiB per page, lane l's 16 bytes landing at base + 16*l,
    // i.e. the page keeps its operand order.  The loads are issued from inline assembly and waited for
    // by hand: they are this wavefront's only vector-memory operations in the main loop.
    bf16_t* ring = reinterpret_cast<bf16_t*>(smem) + (size_t)pgid * RING * 4096;
    const unsigned ring_lds = (unsigned)(size_t)(__attribute__((address_space(3))) void*)ring;
    auto load_page = [&](int slot, int pg) {
        // page ids come through the constant address space: uniform index, so a scalar load that does
        // not enter the vector-memory count
        const int phys = ((const __attribute__((address_space(4))) int32_t*)(uintptr_t)pages)[pg];
        const size_t base = (((size_t)layer * n_pages + phys) * Hkv + g) * (16 * D);
        const bf16_t* kg = k_pool + base + lane * 8;
        const bf16_t* vg = v_pool + base + lane * 8;
#pragma unroll
        for (int c = 0; c < 8; c++) {
            const bf16_t* gp = (c < 4 ? kg : vg) + (c & 3) * 512;
            const unsigned dst = __builtin_amdgcn_readfirstlane(ring_lds + (unsigned)(slot * 8192 + c * 1024));
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gp), "s"(dst) : "memory");
        }
    };
    auto process = [&](int slot, int pg) {
        bf16x8_t kf[4];
        uint4 vraw[4];
        {
            const bf16_t* pb = ring + (size_t)slot * 4096 + lane * 8;
#pragma unroll
            for (int c = 0; c < 4; c++) kf[c] = *reinterpret_cast<const bf16x8_t*>(pb + c * 512);
#pragma unroll
            for (int c = 0; c < 4; c++) vraw[c] = *reinterpret_cast<const uint4*>(pb + 2048 + c * 512);
        }
        const bool need_mask = (pg * 16 + 15) > L;  // page reaches beyond the context: causal part / tail
        float4_t s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks], qf[0][ks], s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks], qf[1][ks], s, 0, 0, 0);
        }
        float sv[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            sv[i] = s[i] * scale_log2;
            if (need_mask) {
                const int tokpos = pg * 16 + lg * 4 + i;
                if (tokpos > L + jrow) sv[i] = -INFINITY;
            }
        }
        float mloc = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
        mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
        // The running reference is kept on whole numbers (scores are in log2 units), so every
        // rescale is an exact power of two and the rounding of p does not depend on the order in
        // which pages are visited: bf16(2^(s-M)) * 2^(M-M') == bf16(2^(s-M')).
        const float mnew = fmaxf(m, ceilf(mloc));
        // the reference moves only on whole numbers, so after the first pages it rarely moves at all:
        // the O accumulators are rescaled only when some row of the tile needs it (wave-uniform test)
        const bool rescale = __builtin_amdgcn_ballot_w64(mnew != m) != 0ull;
        // arguments are <= 0: the bare hardware exponential is enough (results below 2^-126 flush to 0)
        const float alpha = __builtin_amdgcn_exp2f(m - mnew);
        float psum = 0.f;
        short4_t ph, pl;  // p as a bf16 pair
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const float p = __builtin_amdgcn_exp2f(sv[i] - mnew);
            psum += p;
            const __bf16 hi = (__bf16)p;  // round to nearest even, in hardware
            const __bf16 lo = (__bf16)(p - (float)hi);
            ph[i] = __builtin_bit_cast(short, hi);
            pl[i] = __builtin_bit_cast(short, lo);
        }
        lsum = lsum * alpha + psum;
        m = mnew;
        if (rescale) {
#pragma unroll
            for (int dt = 0; dt < 8; dt++)
#pragma unroll
                for (int i = 0; i < 4; i++) o[dt][i] *= alpha;
        }
#pragma unroll
        for (int dt = 0; dt < 8; dt++) {
            // V operand for dims dt*16 .. dt*16+15: half of the 16-byte chunk vraw[dt/2]
            const uint4 r4 = vraw[dt >> 1];
            const uint2 half = (dt & 1) ? make_uint2(r4.z, r4.w) : make_uint2(r4.x, r4.y);
            const short4_t va = __builtin_bit_cast(short4_t, half);
            float4_t acc = o[dt];
            acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va, ph, acc, 0, 0, 0);
            o[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va, pl, acc, 0, 0, 0);
        }
    };

    // Rounds: in round r page group p works on page page0 + p + r*NPG (if the work item has it).
    // The group's producer fetches that page two rounds ahead into ring slot r % RING and waits for it
    // before the barrier that opens round r; after the barrier the consumers may read it -- and they
    // have all finished round r-1, whose slot the fetch issued right after the barrier (for round r+2)
    // overwrites.  Loads retire in order: the page of round r+1 has landed once at most the 8 loads of
    // round r+2 are outstanding.
    constexpr int PF = RING - 1;
    const int n_rounds = (page_end - page0 + NPG - 1) / NPG;                  // uniform over the workgroup
    const int my_rounds = max(0, (page_end - page0 - pgid + NPG - 1) / NPG);  // rounds in which this group has a page
    auto page_of = [&](int r) { return page0 + pgid + r * NPG; };
    // FUSED: pages from the one that holds position L on may contain rows this kernel has just written; they are
    // requested only after the barrier that follows those stores (pages ascend with the round, so the early ones
    // are a prefix of the rounds and the order of issue stays the order of the rounds)
    const int first_new_page = L >> 4;
    if (producer) {
        int issued = 0;
#pragma unroll
        for (int r = 0; r < PF; r++)
            if (r < my_rounds && (!FUSED || page_of(r) < first_new_page)) {
                load_page(r % RING, page_of(r));
                issued = r + 1;
            }
        if (FUSED) {
            __builtin_amdgcn_s_barrier();   // the consumers' K/V stores have been acknowledged (they waited before it)
#pragma unroll
            for (int r = 0; r < PF; r++)
                if (r >= issued && r < my_rounds) load_page(r % RING, page_of(r));
        }
        if (my_rounds > 1)
            asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        else
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        for (int r = 0; r < n_rounds; r++) {
            __builtin_amdgcn_s_barrier();
            if (r + PF < my_rounds) load_page((r + PF) % RING, page_of(r + PF));
            // issued so far: rounds < min(r + PF + 1, my_rounds); the page of round r + 1 is needed next
            if (r + 1 < my_rounds) {
                if (r + 2 < my_rounds)
                    asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
                else
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
        }
    } else {
        if (FUSED) {
            __builtin_amdgcn_s_waitcnt(7 << 4 | 3 << 14 | 15);   // this wavefront's q quads are in LDS ...
            __builtin_amdgcn_s_barrier();   // ... everybody's are, and (s_waitcnt vmcnt(0) above) every new K/V row is in memory
            const bf16_t* qtile = reinterpret_cast<const bf16_t*>(smem) + (size_t)NPG * RING * 4096 + (size_t)qt * 4096 + lane * 8;
#pragma unroll
            for (int pl = 0; pl < 2; pl++)
#pragma unroll
                for (int ks = 0; ks < 4; ks++) qf[pl][ks] = *reinterpret_cast<const bf16x8_t*>(qtile + (pl * 4 + ks) * 512);
        }
        for (int r = 0; r < n_rounds; r++) {
            __builtin_amdgcn_s_waitcnt(7 << 4 | 3 << 14 | 15);  // lgkmcnt(0): this wavefront's LDS reads are back
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            if (active && r < my_rounds) process(r % RING, page_of(r));
            asm volatile("" ::: "memory");
        }
    }
    __syncthreads();  // every page has been consumed, no load is in flight: the rings become the merge buffer

    // lane-partial sums -> per-qrow sums
    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);
    // page groups 1 .. NPG-1 park their states in LDS; group 0 folds them in, in ascending order
    // (exact: every rescale is a power of two)
    float* park = reinterpret_cast<float*>(smem);
    auto fold = [&](float m2, float l2, auto o2_of) {
        const float mnew = fmaxf(m, m2);
        const float a1 = exp2f(m - mnew), a2 = exp2f(m2 - mnew);
        lsum = lsum * a1 + l2 * a2;
        m = mnew;
#pragma unroll
        for (int dt = 0; dt < 8; dt++) {
            const float4_t o2 = o2_of(dt);
#pragma unroll
            for (int i = 0; i < 4; i++) o[dt][i] = o[dt][i] * a1 + o2[i] * a2;
        }
    };
    auto fold_groups = [&]() {  // called by every wavefront that is still alive
        if (!producer && pgid > 0) {
            float* slot = park + (size_t)((pgid - 1) * QT + qt) * ATTN_PARK_F;
            if (lg == 0) {
                slot[2048 + lq] = m;
                slot[2048 + 16 + lq] = lsum;
            }
#pragma unroll
            for (int dt = 0; dt < 8; dt++) *reinterpret_cast<float4_t*>(slot + (dt * 64 + lane) * 4) = o[dt];
        }
        __syncthreads();
        if (!producer && pgid == 0) {
            for (int p2 = 1; p2 < NPG; p2++) {
                const float* slot = park + (size_t)((p2 - 1) * QT + qt) * ATTN_PARK_F;
                fold(slot[2048 + lq], slot[2048 + 16 + lq],
                     [&](int dt) { return *reinterpret_cast<const float4_t*>(slot + (dt * 64 + lane) * 4); });
            }
        }
    };
    fold_groups();

    // The wavefronts of page group 0 now hold the state of work item w, one query tile each.  If the
    // (request, kv head) has several work items, each stores its state; the one that arrives last
    // merges them all in a fixed order (so the result does not depend on which one that is) and writes
    // the output.  Reading a stored state is a round trip to the memory side, so the page groups share
    // the merge: group p takes items p, p + NPG, ... in ascending order, then the groups are folded
    // through LDS as above.
    const int bg = b * Hkv + g;
    const int w0 = rec[8], w1 = rec[9];
    const bool single = (w1 - w0) == 1;
    // Cross-workgroup hand-over without a device-scope fence (which writes back and invalidates a whole
    // L2 and, with one per workgroup, serialises on each XCD): the partial states are written and read
    // with device-scope atomic accesses, which go to the memory-side coherence point themselves, and
    // the arrival counter is bumped only after this workgroup's stores have been acknowledged.
    auto put = [&](float* q4, const float4_t& v) {  // 16 bytes at q4 as two 8-byte coherent stores
        const uint2 a = make_uint2(__float_as_uint(v[0]), __float_as_uint(v[1])), c = make_uint2(__float_as_uint(v[2]), __float_as_uint(v[3]));
        __hip_atomic_store(reinterpret_cast<unsigned long long*>(q4), __builtin_bit_cast(unsigned long long, a), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(reinterpret_cast<unsigned long long*>(q4) + 1, __builtin_bit_cast(unsigned long long, c), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    };
    auto get = [&](const float* q4) {
        const unsigned long long a = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(q4), __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long c = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(q4) + 1, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT);
        const uint2 a2 = __builtin_bit_cast(uint2, a), c2 = __builtin_bit_cast(uint2, c);
        return float4_t{__uint_as_float(a2.x), __uint_as_float(a2.y), __uint_as_float(c2.x), __uint_as_float(c2.y)};
    };
    if (!single) {
        if (!producer && pgid == 0) {
            if (lg == 0) {
                __hip_atomic_store(&part_ml[((size_t)w * 2 + 0) * (QT * 16) + r_mine], m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(&part_ml[((size_t)w * 2 + 1) * (QT * 16) + r_mine], lsum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
#pragma unroll
            for (int dt = 0; dt < 8; dt++) put(part_o + ((size_t)w * (QT * 16) + r_mine) * D + dt * 16 + lg * 4, o[dt]);
            // every store above has been acknowledged before this wavefront reaches the barrier
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_s_waitcnt(0);
        }
        __syncthreads();
        if (tid == 0) {
            const int old = __hip_atomic_fetch_add(&arrive[bg], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int last = old == (w1 - w0 - 1);
            if (last) __hip_atomic_store(&arrive[bg], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next layer
            sh_last = last;
        }
        __syncthreads();
        if (!sh_last || producer) return;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        m = NEG_BIG;
        lsum = 0.f;
#pragma unroll
        for (int dt = 0; dt < 8; dt++) o[dt] = float4_t{0.f, 0.f, 0.f, 0.f};
        for (int ww = w0 + pgid; ww < w1; ww += NPG) {
            const float m2 = __hip_atomic_load(&part_ml[((size_t)ww * 2 + 0) * (QT * 16) + r_mine], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const float l2 = __hip_atomic_load(&part_ml[((size_t)ww * 2 + 1) * (QT * 16) + r_mine], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            fold(m2, l2, [&](int dt) { return get(part_o + ((size_t)ww * (QT * 16) + r_mine) * D + dt * 16 + lg * 4); });
        }
        fold_groups();  // the barrier inside also orders group 0's earlier reads of the parking slots before these writes
        if (pgid != 0) return;
    } else if (producer || pgid != 0) {
        return;
    }
    // normalise and write the attention output as a bf16 pair, in the operand order of the O
    // projection: X[t = row0 + j][col = (g*G + hh)*D + d]; lane holds qrow lq, dims dt*16 + lg*4 + 0..3
    if (r_mine >= rows) return;
    const int Kdim = Hq * D;
    const float inv = 1.0f / lsum;
    const int hh = r_mine - jrow * G;
    const int t = row0 + jrow;
#pragma unroll
    for (int dt = 0; dt < 8; dt++) {
        const int col = (g * G + hh) * D + dt * 16 + lg * 4;
        uint32_t hi2[2], lo2[2];
#pragma unroll
        for (int e = 0; e < 2; e++) {
            const float x0 = o[dt][2 * e] * inv, x1 = o[dt][2 * e + 1] * inv;
            const bf16_t h0 = f32_to_bf16(x0), h1 = f32_to_bf16(x1);
            hi2[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
            lo2[e] = (uint32_t)f32_to_bf16(x0 - bf16_to_f32(h0)) | ((uint32_t)f32_to_bf16(x1 - bf16_to_f32(h1)) << 16);
        }
        const size_t off = frag_offset(t, col, Kdim);
        *reinterpret_cast<uint2*>(X + off) = make_uint2(hi2[0], hi2[1]);
        *reinterpret_cast<uint2*>(X + x_plane + off) = make_uint2(lo2[0], lo2[1]);
    }
}

// fp32 models: one wavefront per (packed row t, query head h); lanes stride over the keys
template <int D>
__global__ __launch_bounds__(64) void attn_f32_kernel(sled_step_meta meta, const int32_t* __restrict__ len_dev,
                                                      const float* __restrict__ Q, const float* __restrict__ k_pool,
                                                      const float* __restrict__ v_pool, int64_t n_pages, int layer, int Hq,
                                                      int Hkv, float scale, float* __restrict__ X) {
    const int t = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const int b = meta.row_req[t], j = meta.row_j[t];
    const int g = h / (Hq / Hkv);
    const int nkeys = len_dev[meta.req_id[b]] + meta.pos0[b] + j + 1;
    const int32_t* pages = meta.pages + meta.cu_pages[b];
    float q[D], o[D];
    const float* qp = Q + ((size_t)t * Hq + h) * D;
#pragma unroll
    for (int d = 0; d < D; d++) {
        q[d] = qp[d];
        o[d] = 0.f;
    }
    float m = NEG_BIG, l = 0.f;
    for (int tok = lane; tok < nkeys; tok += 64) {
        const size_t base = ((((size_t)layer * n_pages + pages[tok >> 4]) * Hkv + g) * 16 + (tok & 15)) * D;
        const float* kp = k_pool + base;
        const float* vp = v_pool + base;
        float s = 0.f;
#pragma unroll
        for (int d = 0; d < D; d++) s = fmaf(q[d], kp[d], s);
        s *= scale;
        const float mnew = fmaxf(m, s);
        const float alpha = expf(m - mnew), p = expf(s - mnew);
        l = l * alpha + p;
#pragma unroll
        for (int d = 0; d < D; d++) o[d] = o[d] * alpha + p * vp[d];
        m = mnew;
    }
    float M = m;
    for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
    const float f = expf(m - M);
    l *= f;
    for (int off = 32; off > 0; off >>= 1) l += __shfl_xor(l, off);
    const float inv = 1.0f / l;
    float* xp = X + (size_t)t * (Hq * D) + h * D;
#pragma unroll
    for (int d = 0; d < D; d++) {
        float v = o[d] * f;
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
        if (lane == (d & 63)) xp[d] = v * inv;
    }
}

}  // namespace

size_t sled_attn_lds_bytes(int QT) {
    const int npg = attn_groups(QT);
    const size_t loop_bytes = (size_t)npg * ATTN_RING * 8192 + (size_t)QT * 8192;                  // page rings, q tiles (fused prologue)
    const size_t merge_bytes = (size_t)(npg - 1) * QT * ATTN_PARK_F * sizeof(float);              // parked states
    return loop_bytes > merge_bytes ? loop_bytes : merge_bytes;
}

int sled_launch_attention(const sled_model* m, const sled_kvpool* p, const sled_step_meta& meta, int layer, const void* Q,
                          size_t q_plane, const float* qkv_partial, int n_split, int T_pad, const float* cs,
                          const int32_t* kvslot, const int32_t* plan, float* part_o, float* part_ml, int32_t* arrive,
                          void* X_out, size_t x_plane, int QT, hipStream_t st) {
    const sled_shape& s = m->s;
    if (s.dtype == SLED_BF16) {
        const float scale_log2 = 1.4426950408889634f / sqrtf((float)s.head_dim);
        const size_t lds = sled_attn_lds_bytes(QT);
        dim3 grid(meta.n_work), blk(64 * (QT + 1) * attn_groups(QT));
        const bool fused = qkv_partial != nullptr;
#define SLED_ATTN_LAUNCH(N, F)                                                                                       \
    {                                                                                                                \
        static bool allowed = false;                                                                                 \
        if (!allowed) {                                                                                              \
            SLED_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bf16_kernel<N, F>),                       \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                     \
            allowed = true;                                                                                          \
        }                                                                                                            \
        hipLaunchKernelGGL((attn_bf16_kernel<N, F>), grid, blk, lds, st, meta, p->len_dev, static_cast<const bf16_t*>(Q), \
                           q_plane, qkv_partial, n_split, T_pad, reinterpret_cast<const float2*>(cs), kvslot, plan,  \
                           static_cast<bf16_t*>(p->k_pool), static_cast<bf16_t*>(p->v_pool), p->n_pages, layer,      \
                           s.n_q_heads, s.n_kv_heads, scale_log2, part_o, part_ml, arrive,                           \
                           static_cast<bf16_t*>(X_out), x_plane);                                                    \
    }
#define SLED_ATTN_CASE(N)                \
    case N:                              \
        if (fused) SLED_ATTN_LAUNCH(N, true) \
        else SLED_ATTN_LAUNCH(N, false)  \
        break;
        switch (QT) {
            SLED_ATTN_CASE(1)
            SLED_ATTN_CASE(2)
            SLED_ATTN_CASE(3)
            SLED_ATTN_CASE(4)
            SLED_ATTN_CASE(5)
            default:
                SLED_FAIL(SLED_EINVAL, "attention: %d query-row tiles unsupported", QT);
        }
#undef SLED_ATTN_CASE
#undef SLED_ATTN_LAUNCH
        SLED_LAUNCH_CHECK();
        return SLED_OK;
    }
    if (qkv_partial) SLED_FAIL(SLED_EINVAL, "attention: the fused QKV prologue exists for bf16 models only");
    const float scale = 1.0f / sqrtf((float)s.head_dim);
    dim3 grid(meta.T, s.n_q_heads);
    if (s.head_dim == 64)
        hipLaunchKernelGGL(attn_f32_kernel<64>, grid, dim3(64), 0, st, meta, p->len_dev, static_cast<const float*>(Q),
                           static_cast<const float*>(p->k_pool), static_cast<const float*>(p->v_pool), p->n_pages, layer,
                           s.n_q_heads, s.n_kv_heads, scale, static_cast<float*>(X_out));
    else if (s.head_dim == 128)
        hipLaunchKernelGGL(attn_f32_kernel<128>, grid, dim3(64), 0, st, meta, p->len_dev, static_cast<const float*>(Q),
                           static_cast<const float*>(p->k_pool), static_cast<const float*>(p->v_pool), p->n_pages, layer,
                           s.n_q_heads, s.n_kv_heads, scale, static_cast<float*>(X_out));
    else
        SLED_FAIL(SLED_EINVAL, "attention: head_dim %d unsupported for fp32 models", s.head_dim);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}
