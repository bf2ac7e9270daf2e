// Projections of the verify step: out[T, N] = X[T, K] * W[N, K]^T over the packed rows of a batch.
//
// bf16 path (the one that matters): T is about 100-600 packed rows, so every weight byte is
// used for only T multiply-adds and the kernel is a weight stream bounded by HBM; it is still a
// dense contraction, so the arithmetic goes through v_mfma_f32_16x16x32_bf16.
//   - Weights sit in HBM in MFMA operand order (see frag_offset): a wavefront fetches a 16-row x
//     32-k tile with one contiguous 1 KiB load straight into registers, no LDS, no transpose, and
//     keeps NBUF-1 pipeline stages of them in flight (HBM latency is covered by bytes in flight per
//     wavefront, not by the number of wavefronts).
//   - Activations are carried as bf16 PAIRS, x = hi + lo (two planes in operand order, written
//     that way by the producing kernel): a single bf16 rounding of every activation costs more
//     accuracy than the 2e-2 logit tolerance allows at 8B scale, while in this HBM-bound regime
//     the MFMA pipes are mostly idle, so each weight tile is multiplied with both planes.
//     They are small and shared by all wavefronts of a workgroup: staged through LDS, double
//     buffered.
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

constexpr int KC = 2;      // k-steps (of 32) per pipeline stage
constexpr int PLANES = 2;  // activation planes: hi, lo

template <int MT, int NW, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const bf16_t* __restrict__ Xp, size_t x_plane,
                                                        const bf16_t* __restrict__ Wp, int NT, int KS, int ks_per_split,
                                                        int T, int T_pad, int N, float* __restrict__ out,
                                                        bf16_t* __restrict__ out_act, size_t act_plane, int F_act) {
    constexpr int NBUF = NW >= 4 ? 3 : 4;  // weight register buffers: the stage in use + the stages in flight
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t* xs = reinterpret_cast<bf16_t*>(smem);  // [2][PLANES][MT][KC][512]
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int nt0 = (blockIdx.x * 4 + wv) * NW;
    const int ks_begin = blockIdx.y * ks_per_split;
    const int ks_end = min(KS, ks_begin + ks_per_split);
    const int n_stage = (ks_end - ks_begin) / KC;
    const int mt_base = blockIdx.z * MT;  // first 16-row tile handled by this block

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
        wbase[a] = Wp + ((size_t)(nt_ok[a] ? nt0 + a : 0) * KS + ks_begin) * 512 + lane * 8;
    }

    // One stage of activations is PLANES*MT*KC KiB = PLANES*MT*KC*64 16-byte pieces over 256 threads.
    constexpr int STAGE_PIECES = PLANES * MT * KC * 64;
    constexpr int XPIECES = (STAGE_PIECES + 255) / 256;
    constexpr int STAGE_ELEMS = PLANES * MT * KC * 512;
    bf16x8_t wreg[NBUF][NW][KC];
    uint4 xreg[XPIECES];

    auto load_w = [&](int buf, int stage) {
#pragma unroll
        for (int a = 0; a < NW; a++)
#pragma unroll
            for (int c = 0; c < KC; c++)
                wreg[buf][a][c] = *reinterpret_cast<const bf16x8_t*>(wbase[a] + (size_t)(stage * KC + c) * 512);
    };
    // piece e of a stage: plane e / (MT*KC*64), row tile, then KC*512 contiguous elements of that
    // tile's k range; LDS keeps the same order
    auto load_x = [&](int stage) {
#pragma unroll
        for (int i = 0; i < XPIECES; i++) {
            const int e = i * 256 + tid;
            if (STAGE_PIECES % 256 == 0 || e < STAGE_PIECES) {
                const int pl = e / (MT * KC * 64), rem = e - pl * (MT * KC * 64);
                const int b = rem / (KC * 64), r = rem - b * (KC * 64);
                xreg[i] = *reinterpret_cast<const uint4*>(Xp + pl * x_plane +
                                                          ((size_t)(mt_base + b) * KS + ks_begin + stage * KC) * 512 + r * 8);
            }
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int i = 0; i < XPIECES; i++) {
            const int e = i * 256 + tid;
            if (STAGE_PIECES % 256 == 0 || e < STAGE_PIECES)
                *reinterpret_cast<uint4*>(xs + (size_t)buf * STAGE_ELEMS + (size_t)e * 8) = xreg[i];
        }
    };
    auto compute = [&](int xbuf, int wbuf) {
#pragma unroll
        for (int c = 0; c < KC; c++) {
#pragma unroll
            for (int b = 0; b < MT; b++) {
                const bf16_t* xp = xs + (size_t)xbuf * STAGE_ELEMS + ((size_t)(b * KC + c)) * 512 + lane * 8;
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

    if (n_stage > 0) {
        // prologue: activations of stage 0 first (they are waited for first), then NBUF-1 weight stages
        load_x(0);
#pragma unroll
        for (int u = 0; u < NBUF - 1; u++)
            if (u < n_stage) load_w(u, u);
        store_x(0);
        __syncthreads();
        constexpr int UNROLL = (NBUF % 2) ? 2 * NBUF : NBUF;  // LDS parity and register buffer both compile-time
        for (int s0 = 0; s0 < n_stage; s0 += UNROLL) {
#pragma unroll
            for (int u = 0; u < UNROLL; u++) {
                const int s = s0 + u;
                if (s < n_stage) {
                    // Loads are issued oldest-needed first: the activation loads of the next stage are
                    // waited for at the end of this stage, the weight loads NBUF-1 stages later, so the
                    // wait on the former leaves the latter in flight.
                    if (s + 1 < n_stage) load_x(s + 1);
                    if (s + NBUF - 1 < n_stage) load_w((u + NBUF - 1) % NBUF, s + NBUF - 1);
                    compute(u & 1, u % NBUF);
                    if (s + 1 < n_stage) store_x((u + 1) & 1);
                    __syncthreads();
                }
            }
        }
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

template <int MT, int NW>
int launch_bf16(int epi, dim3 grid, size_t lds, hipStream_t st, const bf16_t* X, size_t x_plane, const bf16_t* W, int NT,
                int KS, int kps, int T, int T_pad, int N, float* out, bf16_t* out_act, size_t act_plane, int F_act) {
    switch (epi) {
        case SLED_EPI_PARTIAL:
            hipLaunchKernelGGL((gemm_bf16_kernel<MT, NW, SLED_EPI_PARTIAL>), grid, dim3(256), lds, st, X, x_plane, W, NT, KS,
                               kps, T, T_pad, N, out, out_act, act_plane, F_act);
            break;
        case SLED_EPI_SWIGLU:
            hipLaunchKernelGGL((gemm_bf16_kernel<MT, NW, SLED_EPI_SWIGLU>), grid, dim3(256), lds, st, X, x_plane, W, NT, KS,
                               kps, T, T_pad, N, out, out_act, act_plane, F_act);
            break;
        default:
            hipLaunchKernelGGL((gemm_bf16_kernel<MT, NW, SLED_EPI_STORE>), grid, dim3(256), lds, st, X, x_plane, W, NT, KS,
                               kps, T, T_pad, N, out, out_act, act_plane, F_act);
            break;
    }
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

template <int MT>
int launch_bf16_nw(int nw, int epi, dim3 grid, size_t lds, hipStream_t st, const bf16_t* X, size_t x_plane, const bf16_t* W,
                   int NT, int KS, int kps, int T, int T_pad, int N, float* out, bf16_t* out_act, size_t act_plane,
                   int F_act) {
    switch (nw) {
        case 1: return launch_bf16<MT, 1>(epi, grid, lds, st, X, x_plane, W, NT, KS, kps, T, T_pad, N, out, out_act, act_plane, F_act);
        case 2: return launch_bf16<MT, 2>(epi, grid, lds, st, X, x_plane, W, NT, KS, kps, T, T_pad, N, out, out_act, act_plane, F_act);
        default: return launch_bf16<MT, 4>(epi, grid, lds, st, X, x_plane, W, NT, KS, kps, T, T_pad, N, out, out_act, act_plane, F_act);
    }
}

// tuning aid: SLED_GEMM_TUNE="N:K:nw:split;N:K:nw:split;..." overrides the plan of the projections
// with those N and K (read once)
struct tune_entry {
    int N, K, nw, split;
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
            tune_entry te{0, 0, 0, 0};
            if (sscanf(s.substr(pos, end - pos).c_str(), "%d:%d:%d:%d", &te.N, &te.K, &te.nw, &te.split) == 4) v.push_back(te);
            pos = end + 1;
        }
        return v;
    }();
    return t;
}

}  // namespace

// Shape of the launch for a projection of N columns over K: NW 16-column tiles per wavefront and the
// number of K slices.  More tiles per wavefront mean fewer LDS reads per weight byte; more slices
// mean more workgroups (the chip wants at least one per CU) but more partial sums to reduce.
sled_gemm_plan sled_gemm_make_plan(const sled_model* m, int N, int K, bool needs_full_k) {
    sled_gemm_plan p{1, 1};
    if (m->s.dtype != SLED_BF16) return p;
    const int NT = N / 16, stages = K / (32 * KC);
    auto legal_split = [&](int sp) { return sp >= 1 && stages % sp == 0 && (stages / sp) >= 4; };
    for (const auto& te : tune_table())
        if (te.N == N && te.K == K && (te.nw == 1 || te.nw == 2 || te.nw == 4) && legal_split(te.split) &&
            (!needs_full_k || te.split == 1))
            return sled_gemm_plan{te.nw, te.split};
    // default: two tiles per wavefront (128 columns per workgroup); split K until the chip is covered
    p.nw = NT >= 4096 ? 4 : 2;
    const int n_wg = (NT + 4 * p.nw - 1) / (4 * p.nw);
    if (!needs_full_k)
        while (n_wg * p.split < 256 && legal_split(p.split * 2)) p.split *= 2;
    return p;
}

int sled_launch_gemm(const sled_model* m, const void* X, size_t x_plane, const void* W, int T, int T_pad, int N, int K,
                     int epilogue, sled_gemm_plan plan, float* out_f32, void* out_act, size_t act_plane, int F_act,
                     hipStream_t st) {
    if (m->s.dtype == SLED_BF16) {
        if (N % 16 || K % (32 * KC) || T_pad % 16) SLED_FAIL(SLED_EINVAL, "gemm: unsupported shape N=%d K=%d T_pad=%d", N, K, T_pad);
        const int NT = N / 16, KS = K / 32, split_k = plan.split;
        if (KS % split_k || (KS / split_k) % KC) SLED_FAIL(SLED_EINVAL, "gemm: bad split %d for K=%d", split_k, K);
        const int kps = KS / split_k;
        const int mt_total = T_pad / 16;
        // rows are processed in blocks of at most 8 tiles (128 rows), evenly sized
        const int zb = (mt_total + 7) / 8;
        const int MT = (mt_total + zb - 1) / zb;
        const int zblocks = (mt_total + MT - 1) / MT;
        dim3 grid((NT + 4 * plan.nw - 1) / (4 * plan.nw), split_k, zblocks);
        const size_t lds = (size_t)2 * PLANES * MT * KC * 512 * sizeof(bf16_t);
        const bf16_t* Xb = static_cast<const bf16_t*>(X);
        const bf16_t* Wb = static_cast<const bf16_t*>(W);
        bf16_t* oa = static_cast<bf16_t*>(out_act);
#define SLED_GEMM_CASE(M_) \
    case M_:               \
        return launch_bf16_nw<M_>(plan.nw, epilogue, grid, lds, st, Xb, x_plane, Wb, NT, KS, kps, T, T_pad, N, out_f32, oa, act_plane, F_act);
        switch (MT) {
            SLED_GEMM_CASE(1)
            SLED_GEMM_CASE(2)
            SLED_GEMM_CASE(3)
            SLED_GEMM_CASE(4)
            SLED_GEMM_CASE(5)
            SLED_GEMM_CASE(6)
            SLED_GEMM_CASE(7)
            default:
                SLED_GEMM_CASE(8)
        }
#undef SLED_GEMM_CASE
    }
    // fp32: no split, plain store (partial buffer with one slice has the same layout)
    dim3 grid((N + 63) / 64, (T + 15) / 16);
    hipLaunchKernelGGL(gemm_f32_kernel<0>, grid, dim3(256), 0, st, static_cast<const float*>(X),
                       static_cast<const float*>(W), T, N, K, out_f32);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}
