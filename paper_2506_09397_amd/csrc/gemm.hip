// Projections of the verify step: out[T, N] = X[T, K] * W[N, K]^T over the packed rows of a batch.
//
// bf16 path (the one that matters): T is about 100-600 packed rows, so every weight byte is
// used for only T multiply-adds and the kernel is a weight stream bounded by HBM; it is still a
// dense contraction, so the arithmetic goes through v_mfma_f32_16x16x32_bf16.
//   - Weights sit in HBM in MFMA operand order, k-step-major (see wfrag_offset): a wavefront fetches
//     a 16-row x 32-k tile with one contiguous 1 KiB load straight into registers, no LDS, no transpose, and
//     keeps NBUF-1 pipeline stages of them in flight (HBM latency is covered by bytes in flight per
//     wavefront, not by the number of wavefronts).
//   - Activations are carried as bf16 PAIRS, x = hi + lo (two planes in operand order, written
//     that way by the producing kernel): a single bf16 rounding of every activation costs more
//     accuracy than the 2e-2 logit tolerance allows at 8B scale, while in this HBM-bound regime
//     the MFMA pipes are mostly idle, so each weight tile is multiplied with both planes.
//     They are small and shared by all wavefronts of a workgroup: a fifth "producer" wavefront
//     streams them from L2 into a ring of three LDS buffers with direct-to-LDS loads, two stages
//     ahead, while the four "consumer" wavefronts stream weights and do the arithmetic.  The split
//     matters because vector-memory loads retire in order under one counter: a wavefront that
//     issued both kinds could not wait for its activation loads without also draining its weight
//     prefetch.
//   - Each wavefront owns NW 16-column tiles of the output for all rows of its block (MT 16-row
//     tiles): an activation tile read from LDS is reused for NW weight tiles.
//   - Split-K over blockIdx.y gives every CU work on the narrow projections; partial sums go to a
//     [split, T, N] fp32 buffer that the following row kernel reduces in a fixed order (no float
//     atomics: results are reproducible run to run).
//   - The weight tile is the A operand, the activation tile the B operand, so a lane ends up with
//     4 consecutive output columns of one row: float4 stores, and gate/up pairs for SwiGLU in-lane.
//
// fp32 path: plain LDS-tiled FMA kernel, used by fp32 models (correctness configuration).
#include "sled_internal.h"

#include <stdlib.h>
#include <string.h>

namespace {

constexpr int PLANES = 2;  // activation planes: hi, lo
constexpr int NXB = 3;     // LDS ring: the stage being read, the next one (landed), the one after (in flight)
constexpr int NBUF = 4;    // weight register buffers: the stage in use + 3 stages in flight

// s_waitcnt vmcnt(n) alone: expcnt and lgkmcnt fields at their no-wait values
constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

template <int MT, int NW, int KC, int EPI>
__global__ __launch_bounds__(320) void gemm_bf16_kernel(const bf16_t* __restrict__ Xp, size_t x_plane,
                                                        const bf16_t* __restrict__ Wp, int NT, int KS, int ks_per_split,
                                                        int T, int T_pad, int N, float* __restrict__ out,
                                                        bf16_t* __restrict__ out_act, size_t act_plane, int F_act) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t* xs = reinterpret_cast<bf16_t*>(smem);  // [NXB][PLANES][MT][KC][512]
    constexpr int STAGE_TILES = PLANES * MT * KC;  // 1 KiB operand tiles per stage
    constexpr int STAGE_ELEMS = STAGE_TILES * 512;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int ks_begin = blockIdx.y * ks_per_split;
    const int n_stage = ks_per_split / KC;  // a positive multiple of NBUF (the host picks K slices accordingly)
    const int mt_base = blockIdx.z * MT;    // first 16-row tile handled by this block

    if (wv == 4) {
        // ---- producer wavefront: activations L2 -> LDS, two stages ahead of the consumers -------
        // One direct-to-LDS load moves a whole operand tile: lane l's 16 bytes land at base + 16*l.
        auto dma = [&](int buf, int stage) {
#pragma unroll
            for (int i = 0; i < STAGE_TILES; i++) {
                const int pl = i / (MT * KC), rem = i - pl * (MT * KC);
                const int b = rem / KC, c = rem - b * KC;
                const bf16_t* g = Xp + pl * x_plane + ((size_t)(mt_base + b) * KS + ks_begin + stage * KC + c) * 512 + lane * 8;
                bf16_t* l = xs + (size_t)buf * STAGE_ELEMS + (size_t)i * 512;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                                 (__attribute__((address_space(3))) void*)l, 16, 0, 0);
            }
        };
        dma(0, 0);
        dma(1, 1);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(STAGE_TILES));  // stage 0 has landed, stage 1 may be in flight
        __builtin_amdgcn_s_barrier();
        int buf = 2;
        for (int s = 0; s < n_stage; s++) {
            // buffer `buf` held stage s-1: its readers passed the previous barrier
            if (s + 2 < n_stage) {
                dma(buf, s + 2);
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(STAGE_TILES));  // loads retire in order: stage s+1 has landed
            } else {
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            }
            __builtin_amdgcn_s_barrier();  // publishes stage s+1, and says stage s has been consumed
            buf = buf == NXB - 1 ? 0 : buf + 1;
        }
        return;
    }

    // ---- consumer wavefronts: weights HBM -> registers, MFMA ---------------------------------------
    const int nt0 = (blockIdx.x * 4 + wv) * NW;
    float4_t acc[NW][MT];
#pragma unroll
    for (int a = 0; a < NW; a++)
#pragma unroll
        for (int b = 0; b < MT; b++) acc[a][b] = float4_t{0.f, 0.f, 0.f, 0.f};

    bool nt_ok[NW];
    const bf16_t* wbase[NW];
#pragma unroll
    for (int a = 0; a < NW; a++) {
        nt_ok[a] = (nt0 + a) < NT;
        wbase[a] = Wp + ((size_t)ks_begin * NT + (nt_ok[a] ? nt0 + a : 0)) * 512 + lane * 8;
    }
    bf16x8_t wreg[NBUF][NW][KC];
    auto load_w = [&](int buf, int stage) {
#pragma unroll
        for (int a = 0; a < NW; a++)
#pragma unroll
            for (int c = 0; c < KC; c++)
                wreg[buf][a][c] = *reinterpret_cast<const bf16x8_t*>(wbase[a] + (size_t)(stage * KC + c) * NT * 512);
    };
    auto compute = [&](const bf16_t* xb, int wbuf) {
#pragma unroll
        for (int c = 0; c < KC; c++) {
#pragma unroll
            for (int b = 0; b < MT; b++) {
                const bf16_t* xp = xb + ((size_t)(b * KC + c)) * 512 + lane * 8;
                const bf16x8_t xhi = *reinterpret_cast<const bf16x8_t*>(xp);
                const bf16x8_t xlo = *reinterpret_cast<const bf16x8_t*>(xp + MT * KC * 512);
#pragma unroll
                for (int a = 0; a < NW; a++) {
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wreg[wbuf][a][c], xhi, acc[a][b], 0, 0, 0);
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wreg[wbuf][a][c], xlo, acc[a][b], 0, 0, 0);
                }
            }
        }
    };

#pragma unroll
    for (int u = 0; u < NBUF - 1; u++) load_w(u, u);
    __builtin_amdgcn_s_barrier();  // stage 0 of the activations is in LDS
    int xbuf = 0;
    // NBUF stages per trip so that the weight register buffer is a compile-time index.  The only
    // vector-memory operations of these wavefronts are the weight loads, so the compiler's own wait
    // before a stage's arithmetic leaves the three later stages in flight.
    // All trips but the last prefetch unconditionally; the last one has nothing left to fetch after
    // its first stage.  Keeping run-time conditions out of the trips matters: the compiler sizes
    // each wait for the path with the fewest loads outstanding.
    int s0 = 0;
    for (; s0 + NBUF < n_stage; s0 += NBUF) {
#pragma unroll
        for (int u = 0; u < NBUF; u++) {
            load_w((u + NBUF - 1) % NBUF, s0 + u + NBUF - 1);
            __builtin_amdgcn_sched_barrier(0);
            compute(xs + (size_t)xbuf * STAGE_ELEMS, u);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
            xbuf = xbuf == NXB - 1 ? 0 : xbuf + 1;
        }
    }
#pragma unroll
    for (int u = 0; u < NBUF; u++) {
        if (u == 0) load_w(NBUF - 1, s0 + NBUF - 1);
        __builtin_amdgcn_sched_barrier(0);
        compute(xs + (size_t)xbuf * STAGE_ELEMS, u);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        xbuf = xbuf == NXB - 1 ? 0 : xbuf + 1;
    }

    // epilogue: lane holds rows (tokens) mt*16 + lane%16, columns nt*16 + (lane/16)*4 + 0..3
    const int col_in_tile = (lane >> 4) * 4;
#pragma unroll
    for (int a = 0; a < NW; a++) {
        if (!nt_ok[a]) continue;
        const int n = (nt0 + a) * 16 + col_in_tile;
#pragma unroll
        for (int b = 0; b < MT; b++) {
            const int tok = (mt_base + b) * 16 + (lane & 15);
            if (EPI == SLED_EPI_PARTIAL) {
                if (tok < T_pad)
                    *reinterpret_cast<float4_t*>(out + ((size_t)blockIdx.y * T_pad + tok) * N + n) = acc[a][b];
            } else if (EPI == SLED_EPI_STORE) {
                if (tok < T) *reinterpret_cast<float4_t*>(out + (size_t)tok * N + n) = acc[a][b];
            } else {  // SwiGLU: columns are (gate f, up f, gate f+1, up f+1)
                if (tok < T_pad) {
                    const int f = n >> 1;
                    float g0 = acc[a][b][0], u0 = acc[a][b][1], g1 = acc[a][b][2], u1 = acc[a][b][3];
                    float a0 = g0 / (1.f + __expf(-g0)) * u0;
                    float a1 = g1 / (1.f + __expf(-g1)) * u1;
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
    int NT, KS, kps, T, T_pad, N;
    float* out;
    bf16_t* out_act;
    size_t act_plane;
    int F_act;
};

template <int MT, int NW, int KC, int EPI>
int launch_one(const gemm_args& a) {
    // more than 64 KiB of dynamic LDS has to be allowed once per kernel
    static bool allowed = false;
    auto kern = gemm_bf16_kernel<MT, NW, KC, EPI>;
    if (!allowed) {
        SLED_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)a.lds));
        allowed = true;
    }
    hipLaunchKernelGGL(kern, a.grid, dim3(320), a.lds, a.st, a.X, a.x_plane, a.W, a.NT, a.KS, a.kps, a.T, a.T_pad, a.N,
                       a.out, a.out_act, a.act_plane, a.F_act);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

template <int MT, int NW, int KC>
int launch_epi(int epi, const gemm_args& a) {
    switch (epi) {
        case SLED_EPI_PARTIAL: return launch_one<MT, NW, KC, SLED_EPI_PARTIAL>(a);
        case SLED_EPI_SWIGLU: return launch_one<MT, NW, KC, SLED_EPI_SWIGLU>(a);
        default: return launch_one<MT, NW, KC, SLED_EPI_STORE>(a);
    }
}

template <int MT>
int launch_cfg(int nw, int kc, int epi, const gemm_args& a) {
    if (kc == 1) {
        switch (nw) {
            case 1: return launch_epi<MT, 1, 1>(epi, a);
            case 2: return launch_epi<MT, 2, 1>(epi, a);
            default: return launch_epi<MT, 4, 1>(epi, a);
        }
    }
    switch (nw) {
        case 1: return launch_epi<MT, 1, 2>(epi, a);
        case 2: return launch_epi<MT, 2, 2>(epi, a);
        default: return launch_epi<MT, 4, 2>(epi, a);
    }
}

// tuning aid: SLED_GEMM_TUNE="N:K:nw:kc:split;..." overrides the plan of the projections with those
// N and K (read once)
struct tune_entry {
    int N, K, nw, kc, split;
};
const std::vector<tune_entry>& tune_table() {
    static std::vector<tune_entry> t = [] {
        std::vector<tune_entry> v;
        const char* e = getenv("SLED_GEMM_TUNE");
        if (!e) return v;
        std::string s(e);
        size_t pos = 0;
        while (pos < s.size()) {
            size_t end = s.find(';', pos);
            if (end == std::string::npos) end = s.size();
            tune_entry te{0, 0, 0, 0, 0};
            if (sscanf(s.substr(pos, end - pos).c_str(), "%d:%d:%d:%d:%d", &te.N, &te.K, &te.nw, &te.kc, &te.split) == 5)
                v.push_back(te);
            pos = end + 1;
        }
        return v;
    }();
    return t;
}

}  // namespace

// Shape of the launch for a projection of N columns over K: NW 16-column tiles per wavefront, KC
// k-steps per pipeline stage and the number of K slices.  More tiles per wavefront mean fewer LDS
// reads per weight byte; more slices mean more workgroups (the chip wants at least one per CU) but
// more partial sums to reduce.  Each slice must hold a multiple of 4 stages.
sled_gemm_plan sled_gemm_make_plan(const sled_model* m, int N, int K, bool needs_full_k) {
    sled_gemm_plan p{1, 1, 1};
    if (m->s.dtype != SLED_BF16) return p;
    const int NT = N / 16;
    auto legal = [&](int kc, int sp) { return sp >= 1 && (K / 32) % (sp * kc * NBUF) == 0; };
    for (const auto& te : tune_table())
        if (te.N == N && te.K == K && (te.nw == 1 || te.nw == 2 || te.nw == 4) && (te.kc == 1 || te.kc == 2) &&
            legal(te.kc, te.split) && (!needs_full_k || te.split == 1))
            return sled_gemm_plan{te.nw, te.kc, te.split};
    p.nw = NT >= 4096 ? 4 : 2;
    p.kc = 1;
    const int n_wg = (NT + 4 * p.nw - 1) / (4 * p.nw);
    if (!needs_full_k)
        while (n_wg * p.split < 256 && legal(p.kc, p.split * 2)) p.split *= 2;
    return p;
}

int sled_launch_gemm(const sled_model* m, const void* X, size_t x_plane, const void* W, int T, int T_pad, int N, int K,
                     int epilogue, sled_gemm_plan plan, float* out_f32, void* out_act, size_t act_plane, int F_act,
                     hipStream_t st) {
    if (m->s.dtype == SLED_BF16) {
        const int NT = N / 16, KS = K / 32;
        if (N % 16 || K % 32 || T_pad % 16 || KS % (plan.split * plan.kc * NBUF))
            SLED_FAIL(SLED_EINVAL, "gemm: unsupported shape N=%d K=%d T_pad=%d split=%d kc=%d", N, K, T_pad, plan.split, plan.kc);
        const int mt_total = T_pad / 16;
        // rows are processed in blocks of at most 8 tiles (128 rows), evenly sized
        const int zb = (mt_total + 7) / 8;
        const int MT = (mt_total + zb - 1) / zb;
        gemm_args a;
        a.grid = dim3((NT + 4 * plan.nw - 1) / (4 * plan.nw), plan.split, (mt_total + MT - 1) / MT);
        a.lds = (size_t)NXB * PLANES * MT * plan.kc * 512 * sizeof(bf16_t);
        a.st = st;
        a.X = static_cast<const bf16_t*>(X);
        a.x_plane = x_plane;
        a.W = static_cast<const bf16_t*>(W);
        a.NT = NT;
        a.KS = KS;
        a.kps = KS / plan.split;
        a.T = T;
        a.T_pad = T_pad;
        a.N = N;
        a.out = out_f32;
        a.out_act = static_cast<bf16_t*>(out_act);
        a.act_plane = act_plane;
        a.F_act = F_act;
        switch (MT) {
            case 1: return launch_cfg<1>(plan.nw, plan.kc, epilogue, a);
            case 2: return launch_cfg<2>(plan.nw, plan.kc, epilogue, a);
            case 3: return launch_cfg<3>(plan.nw, plan.kc, epilogue, a);
            case 4: return launch_cfg<4>(plan.nw, plan.kc, epilogue, a);
            case 5: return launch_cfg<5>(plan.nw, plan.kc, epilogue, a);
            case 6: return launch_cfg<6>(plan.nw, plan.kc, epilogue, a);
            case 7: return launch_cfg<7>(plan.nw, plan.kc, epilogue, a);
            default: return launch_cfg<8>(plan.nw, plan.kc, epilogue, a);
        }
    }
    // fp32: no split, plain store (partial buffer with one slice has the same layout)
    dim3 grid((N + 63) / 64, (T + 15) / 16);
    hipLaunchKernelGGL(gemm_f32_kernel<0>, grid, dim3(256), 0, st, static_cast<const float*>(X),
                       static_cast<const float*>(W), T, N, K, out_f32);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}
