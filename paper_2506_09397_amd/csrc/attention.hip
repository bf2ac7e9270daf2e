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
// first product and V for the second, so a wavefront moves a whole page with 4 + 4 contiguous
// 1 KiB direct-to-LDS loads into its private ring of three page buffers, two pages in flight while one
// is consumed.  The four wavefronts of a workgroup take alternate pages and merge their (max, sum, O)
// states through LDS at the end.  When a
// (request, kv head) is split over several work items, each stores its state and the last one to
// arrive (a device-scope counter) merges them in a fixed order; either way the output is written in
// the operand order of the following projection, as a bf16 pair.
//
// fp32 kernel (fp32 models): one wavefront per (row, query head), lanes over keys.
#include "sled_internal.h"

namespace {

constexpr float NEG_BIG = -1.0e30f;

constexpr int ATTN_WAVES = 4;  // wavefronts per workgroup: one per SIMD, each with the whole register file

// LDS merge slots: floats per slot = O tile + max + sum
__host__ __device__ constexpr int attn_slot_floats(int QT) { return QT * 8 * 64 * 4 + 2 * QT * 16; }
__host__ __device__ constexpr int attn_slots(int QT) { return QT <= 5 ? 2 : 1; }

template <int QT>
__global__ __launch_bounds__(64 * ATTN_WAVES) __attribute__((amdgpu_waves_per_eu(1, 1))) void attn_bf16_kernel(
    sled_step_meta meta, const int32_t* __restrict__ len_dev, const bf16_t* __restrict__ Q, size_t q_plane,
    const bf16_t* __restrict__ k_pool, const bf16_t* __restrict__ v_pool, int64_t n_pages, int layer, int Hq, int Hkv,
    float scale_log2, float* __restrict__ part_o, float* __restrict__ part_ml, int32_t* __restrict__ arrive,
    bf16_t* __restrict__ X, size_t x_plane) {
    constexpr int D = 128;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // main loop: Q operand tiles [2 planes][QT][4 k-steps][64 lanes][8] (the size of one O tile);
    // afterwards the same bytes serve as merge slots
    bf16_t* sh_q = reinterpret_cast<bf16_t*>(smem);
    float* sh_f = reinterpret_cast<float*>(smem);
    __shared__ int sh_last;

    const int w = blockIdx.x;
    const int b = meta.work[4 * w + 0], g = meta.work[4 * w + 1];
    const int page0 = meta.work[4 * w + 2], npg = meta.work[4 * w + 3];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: page ids are then fetched by scalar loads
    const int G = Hq / Hkv;
    const int L = len_dev[meta.req_id[b]];
    const int n = meta.k[b] + 1;
    const int rows = G * n;
    const int row0 = meta.cu_rows[b];
    const int n_valid_pages = (L + n + 15) >> 4;
    const int page_end = min(page0 + npg, n_valid_pages);
    const int32_t* pages = meta.pages + meta.cu_pages[b];
    const int lq = lane & 15, lg = lane >> 4;

    // Q operand tiles, both planes of the bf16 pair: qrow r = qt*16 + l%16 -> (query position
    // j = r / G, head g*G + r % G); element k = ks*32 + (l/16)*8 ..+8
    for (int e = tid; e < 2 * QT * 4 * 64; e += 64 * ATTN_WAVES) {
        const int l = e & 63, ks = (e >> 6) & 3, qt = (e >> 8) % QT, pl = e / (QT * 256);
        const int r = qt * 16 + (l & 15);
        uint4 val = make_uint4(0u, 0u, 0u, 0u);
        if (r < rows) {
            const int j = r / G, hh = r - j * G;
            val = *reinterpret_cast<const uint4*>(Q + pl * q_plane + ((size_t)(row0 + j) * Hq + g * G + hh) * D + ks * 32 +
                                                  (l >> 4) * 8);
        }
        *reinterpret_cast<uint4*>(sh_q + (size_t)e * 8) = val;
    }
    __syncthreads();
    int jrow[QT];
#pragma unroll
    for (int qt = 0; qt < QT; qt++) jrow[qt] = (qt * 16 + lq) / G;
    // every wavefront keeps the whole Q operand in registers (one wavefront per SIMD owns the full
    // register file): the main loop's LDS traffic is then the K/V pages alone
    // (up to 48 query rows; larger tiles would spill and keep reading Q from LDS)
    constexpr bool Q_IN_REGS = QT <= 3;
    bf16x8_t qreg[2][Q_IN_REGS ? QT : 1][4];
    if (Q_IN_REGS) {
#pragma unroll
        for (int pl = 0; pl < 2; pl++)
#pragma unroll
            for (int qt = 0; qt < QT; qt++)
#pragma unroll
                for (int ks = 0; ks < 4; ks++)
                    qreg[pl][qt][ks] = *reinterpret_cast<const bf16x8_t*>(sh_q + ((size_t)((pl * QT + qt) * 4 + ks) * 64 + lane) * 8);
    }

    float m[QT], lsum[QT];
    float4_t o[QT][8];
#pragma unroll
    for (int qt = 0; qt < QT; qt++) {
        m[qt] = NEG_BIG;
        lsum[qt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < 8; dt++) o[qt][dt] = float4_t{0.f, 0.f, 0.f, 0.f};
    }

    // K/V pages go from HBM straight into a private LDS ring of this wavefront (RING pages of 8 KiB:
    // the one being consumed and the ones in flight) with direct-to-LDS loads: 4 + 4 loads of 1 KiB
    // per page, lane l's 16 bytes landing at base + 16*l, i.e. the page keeps its operand order.
    // The loads are issued from inline assembly and waited for by hand: they are the only
    // vector-memory operations of the main loop, loads retire in order, so "at most 8*n
    // outstanding" means every page but the last n issued has landed.
    constexpr int RING = 3;
    bf16_t* ring = sh_q + (size_t)QT * 4096 + (size_t)wv * RING * 4096;  // after the Q tiles
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
    struct page_regs {
        bf16x8_t kf[4];
        uint4 vraw[4];
    };
    auto process = [&](int slot, int pg) {
        page_regs pr;
        {
            const bf16_t* pb = ring + (size_t)slot * 4096 + lane * 8;
#pragma unroll
            for (int c = 0; c < 4; c++) pr.kf[c] = *reinterpret_cast<const bf16x8_t*>(pb + c * 512);
#pragma unroll
            for (int c = 0; c < 4; c++) pr.vraw[c] = *reinterpret_cast<const uint4*>(pb + 2048 + c * 512);
        }
        const bool need_mask = (pg * 16 + 15) > L;  // page reaches beyond the context: causal part / tail
#pragma unroll
        for (int qt = 0; qt < QT; qt++) {
            float4_t s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ks++) {
                bf16x8_t qh, ql;
                if (Q_IN_REGS) {
                    qh = qreg[0][qt][ks];
                    ql = qreg[1][qt][ks];
                } else {
                    qh = *reinterpret_cast<const bf16x8_t*>(sh_q + ((size_t)(qt * 4 + ks) * 64 + lane) * 8);
                    ql = *reinterpret_cast<const bf16x8_t*>(sh_q + ((size_t)((QT + qt) * 4 + ks) * 64 + lane) * 8);
                }
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pr.kf[ks], qh, s, 0, 0, 0);
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pr.kf[ks], ql, s, 0, 0, 0);
            }
            float sv[4];
#pragma unroll
            for (int i = 0; i < 4; i++) {
                sv[i] = s[i] * scale_log2;
                if (need_mask) {
                    const int tokpos = pg * 16 + lg * 4 + i;
                    if (tokpos > L + jrow[qt]) sv[i] = -INFINITY;
                }
            }
            float mloc = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
            mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
            mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
            // The running reference is kept on whole numbers (scores are in log2 units), so every
            // rescale is an exact power of two and the rounding of p does not depend on the order in
            // which pages are visited: bf16(2^(s-M)) * 2^(M-M') == bf16(2^(s-M')).
            const float mnew = fmaxf(m[qt], ceilf(mloc));
            // the reference moves only on whole numbers, so after the first pages it rarely moves at all:
            // the O accumulators are rescaled only when some row of the tile needs it (wave-uniform test)
            const bool rescale = __builtin_amdgcn_ballot_w64(mnew != m[qt]) != 0ull;
            // arguments are <= 0: the bare hardware exponential is enough (results below 2^-126 flush to 0)
            const float alpha = __builtin_amdgcn_exp2f(m[qt] - mnew);
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
            lsum[qt] = lsum[qt] * alpha + psum;
            m[qt] = mnew;
            if (rescale) {
#pragma unroll
                for (int dt = 0; dt < 8; dt++)
#pragma unroll
                    for (int i = 0; i < 4; i++) o[qt][dt][i] *= alpha;
            }
#pragma unroll
            for (int dt = 0; dt < 8; dt++) {
                // V operand for dims dt*16 .. dt*16+15: half of the 16-byte chunk vraw[dt/2]
                const uint4 r4 = pr.vraw[dt >> 1];
                const uint32_t lo = (dt & 1) ? r4.z : r4.x, hi = (dt & 1) ? r4.w : r4.y;
                short4_t va;
                va[0] = (short)(lo & 0xffff);
                va[1] = (short)(lo >> 16);
                va[2] = (short)(hi & 0xffff);
                va[3] = (short)(hi >> 16);
                float4_t acc = o[qt][dt];
                acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va, ph, acc, 0, 0, 0);
                o[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va, pl, acc, 0, 0, 0);
            }
        }
    };

    // the wavefront's pages page0 + wv, + ATTN_WAVES, ...: two in flight while one is consumed
    {
        const int first = page0 + wv;
        const int n_my = first < page_end ? (page_end - first + ATTN_WAVES - 1) / ATTN_WAVES : 0;
        if (n_my > 0) load_page(0, first);
        if (n_my > 1) load_page(1, first + ATTN_WAVES);
        int slot = 0, slot2 = 2;
        for (int i = 0; i < n_my; i++) {
            // slot2 held page i-1, whose LDS reads have been consumed by the arithmetic above
            if (i + 2 < n_my) {
                load_page(slot2, first + (i + 2) * ATTN_WAVES);
                __builtin_amdgcn_s_waitcnt((16 & 15) | (7 << 4) | (15 << 8) | ((16 >> 4) << 14));  // vmcnt(16): page i has landed
            } else if (i + 1 < n_my) {
                __builtin_amdgcn_s_waitcnt(8 | (7 << 4) | (15 << 8));
            } else {
                __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));
            }
            asm volatile("" ::: "memory");
            process(slot, first + i * ATTN_WAVES);
            asm volatile("" ::: "memory");
            slot = slot == RING - 1 ? 0 : slot + 1;
            slot2 = slot2 == RING - 1 ? 0 : slot2 + 1;
        }
    }
    __syncthreads();  // all wavefronts are done with the Q tiles: the bytes become the merge buffer
    // lane-partial sums -> per-qrow sums
#pragma unroll
    for (int qt = 0; qt < QT; qt++) {
        lsum[qt] += __shfl_xor(lsum[qt], 16);
        lsum[qt] += __shfl_xor(lsum[qt], 32);
    }
    // merge the wavefronts' states pairwise through LDS: 4 -> 2 -> 1 (exact: every rescale is
    // a power of two), at most attn_slots(QT) writers at a time
    auto merge_from = [&](const float* slot) {
#pragma unroll
        for (int qt = 0; qt < QT; qt++) {
            const float m2 = slot[QT * 2048 + qt * 16 + lq], l2 = slot[QT * 2048 + QT * 16 + qt * 16 + lq];
            const float mnew = fmaxf(m[qt], m2);
            const float a1 = exp2f(m[qt] - mnew), a2 = exp2f(m2 - mnew);
            lsum[qt] = lsum[qt] * a1 + l2 * a2;
            m[qt] = mnew;
#pragma unroll
            for (int dt = 0; dt < 8; dt++) {
                const float4_t o2 = *reinterpret_cast<const float4_t*>(slot + ((qt * 8 + dt) * 64 + lane) * 4);
#pragma unroll
                for (int i = 0; i < 4; i++) o[qt][dt][i] = o[qt][dt][i] * a1 + o2[i] * a2;
            }
        }
    };
    auto store_to = [&](float* slot) {
#pragma unroll
        for (int qt = 0; qt < QT; qt++) {
            if (lg == 0) {
                slot[QT * 2048 + qt * 16 + lq] = m[qt];
                slot[QT * 2048 + QT * 16 + qt * 16 + lq] = lsum[qt];
            }
#pragma unroll
            for (int dt = 0; dt < 8; dt++) *reinterpret_cast<float4_t*>(slot + ((qt * 8 + dt) * 64 + lane) * 4) = o[qt][dt];
        }
    };
    constexpr int SLOTS = attn_slots(QT), SLOT_F = attn_slot_floats(QT);
#pragma unroll
    for (int half = ATTN_WAVES / 2; half >= 1; half >>= 1) {
        for (int g0 = 0; g0 < half; g0 += SLOTS) {
            // wavefronts half+g0 .. half+g0+SLOTS-1 hand their state to wavefronts g0 .. g0+SLOTS-1
            if (wv >= half + g0 && wv < half + g0 + SLOTS && wv < 2 * half) store_to(sh_f + (size_t)(wv - half - g0) * SLOT_F);
            __syncthreads();
            if (wv >= g0 && wv < g0 + SLOTS && wv < half) merge_from(sh_f + (size_t)(wv - g0) * SLOT_F);
            __syncthreads();
        }
    }

    // Wavefront 0 now holds the state of work item w.  If the (request, kv head) has several work
    // items, each stores its state; the one that arrives last merges them all in ascending order
    // (so the result does not depend on which one that is) and writes the output.
    const int bg = b * Hkv + g;
    const int w0 = meta.cu_work[bg], w1 = meta.cu_work[bg + 1];
    const bool single = (w1 - w0) == 1;
    if (!single) {
        if (wv == 0) {
#pragma unroll
            for (int qt = 0; qt < QT; qt++) {
                const int r = qt * 16 + lq;
                if (lg == 0) {
                    part_ml[((size_t)w * 2 + 0) * (QT * 16) + r] = m[qt];
                    part_ml[((size_t)w * 2 + 1) * (QT * 16) + r] = lsum[qt];
                }
#pragma unroll
                for (int dt = 0; dt < 8; dt++)
                    *reinterpret_cast<float4_t*>(part_o + ((size_t)w * (QT * 16) + r) * D + dt * 16 + lg * 4) = o[qt][dt];
            }
            __threadfence();  // the stores above are visible device-wide before the arrival is counted
            if (lane == 0) {
                const int old = atomicAdd(&arrive[bg], 1);
                const int last = old == (w1 - w0 - 1);
                if (last) arrive[bg] = 0;  // ready for the next layer
                sh_last = last;
            }
        }
        __syncthreads();
        if (!sh_last) return;
        if (wv != 0) return;
        __threadfence();  // see the other work items' stores
#pragma unroll
        for (int qt = 0; qt < QT; qt++) {
            m[qt] = NEG_BIG;
            lsum[qt] = 0.f;
#pragma unroll
            for (int dt = 0; dt < 8; dt++) o[qt][dt] = float4_t{0.f, 0.f, 0.f, 0.f};
        }
        for (int ww = w0; ww < w1; ww++) {
#pragma unroll
            for (int qt = 0; qt < QT; qt++) {
                const int r = qt * 16 + lq;
                const float m2 = part_ml[((size_t)ww * 2 + 0) * (QT * 16) + r];
                const float l2 = part_ml[((size_t)ww * 2 + 1) * (QT * 16) + r];
                const float mnew = fmaxf(m[qt], m2);
                const float a1 = exp2f(m[qt] - mnew), a2 = exp2f(m2 - mnew);
                lsum[qt] = lsum[qt] * a1 + l2 * a2;
                m[qt] = mnew;
#pragma unroll
                for (int dt = 0; dt < 8; dt++) {
                    const float4_t o2 = *reinterpret_cast<const float4_t*>(part_o + ((size_t)ww * (QT * 16) + r) * D + dt * 16 + lg * 4);
#pragma unroll
                    for (int i = 0; i < 4; i++) o[qt][dt][i] = o[qt][dt][i] * a1 + o2[i] * a2;
                }
            }
        }
    } else if (wv != 0) {
        return;
    }
    // normalise and write the attention output as a bf16 pair, in the operand order of the O
    // projection: X[t = row0 + j][col = (g*G + hh)*D + d]; lane holds qrow lq, dims dt*16 + lg*4 + 0..3
    const int Kdim = Hq * D;
#pragma unroll
    for (int qt = 0; qt < QT; qt++) {
        const int r = qt * 16 + lq;
        if (r >= rows) continue;
        const float inv = 1.0f / lsum[qt];
        const int j = r / G, hh = r - j * G;
        const int t = row0 + j;
#pragma unroll
        for (int dt = 0; dt < 8; dt++) {
            const int col = (g * G + hh) * D + dt * 16 + lg * 4;
            uint32_t hi2[2], lo2[2];
#pragma unroll
            for (int e = 0; e < 2; e++) {
                const float x0 = o[qt][dt][2 * e] * inv, x1 = o[qt][dt][2 * e + 1] * inv;
                const bf16_t h0 = f32_to_bf16(x0), h1 = f32_to_bf16(x1);
                hi2[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
                lo2[e] = (uint32_t)f32_to_bf16(x0 - bf16_to_f32(h0)) | ((uint32_t)f32_to_bf16(x1 - bf16_to_f32(h1)) << 16);
            }
            const size_t off = frag_offset(t, col, Kdim);
            *reinterpret_cast<uint2*>(X + off) = make_uint2(hi2[0], hi2[1]);
            *reinterpret_cast<uint2*>(X + x_plane + off) = make_uint2(lo2[0], lo2[1]);
        }
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
    const int nkeys = len_dev[meta.req_id[b]] + j + 1;
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
    const size_t loop_bytes = (size_t)QT * 8192 + (size_t)ATTN_WAVES * 3 * 8192;  // Q tiles + per-wavefront page rings
    const size_t merge_bytes = (size_t)attn_slots(QT) * attn_slot_floats(QT) * sizeof(float);
    return loop_bytes > merge_bytes ? loop_bytes : merge_bytes;
}

int sled_launch_attention(const sled_model* m, const sled_kvpool* p, const sled_step_meta& meta, int layer, const void* Q,
                          size_t q_plane, float* part_o, float* part_ml, int32_t* arrive, void* X_out, size_t x_plane,
                          int QT, hipStream_t st) {
    const sled_shape& s = m->s;
    if (s.dtype == SLED_BF16) {
        const float scale_log2 = 1.4426950408889634f / sqrtf((float)s.head_dim);
        const size_t lds = sled_attn_lds_bytes(QT);
        dim3 grid(meta.n_work), blk(64 * ATTN_WAVES);
#define SLED_ATTN_CASE(N)                                                                                            \
    case N: {                                                                                                        \
        static bool allowed = false;                                                                                 \
        if (!allowed) {                                                                                              \
            SLED_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bf16_kernel<N>),                          \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                     \
            allowed = true;                                                                                          \
        }                                                                                                            \
        hipLaunchKernelGGL(attn_bf16_kernel<N>, grid, blk, lds, st, meta, p->len_dev, static_cast<const bf16_t*>(Q),  \
                           q_plane, static_cast<const bf16_t*>(p->k_pool), static_cast<const bf16_t*>(p->v_pool),     \
                           p->n_pages, layer, s.n_q_heads, s.n_kv_heads, scale_log2, part_o, part_ml, arrive,         \
                           static_cast<bf16_t*>(X_out), x_plane);                                                    \
    } break;
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
        SLED_LAUNCH_CHECK();
        return SLED_OK;
    }
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
