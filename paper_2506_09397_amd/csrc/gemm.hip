// Projections of the verify step: out[T, N] = X[T, K] * W[N, K]^T over the packed rows of a batch.
//
// bf16 path (the one that matters): T is about 100-600 packed rows, so every weight byte is
// used for only T multiply-adds and the kernel is a weight stream bounded by HBM; it is still a
// dense contraction, so the arithmetic goes through v_mfma_f32_16x16x32_bf16.
//   - Weights sit in HBM in MFMA operand order (see frag_offset): a wavefront fetches a 16-row x
//     32-k tile with one contiguous 1 KiB load straight into registers, no LDS, no transpose.
//   - Activations (also in operand order, written that way by the producing kernel) are small and
//     shared by all wavefronts of a workgroup: they are staged through LDS, double buffered.
//   - Each wavefront owns NW 16-column tiles of the output for all T rows (MT 16-row tiles), so a
//     weight byte is read exactly once per 128 rows.
//   - Split-K over blockIdx.y gives every CU work on the narrow projections; partial sums go to a
//     [split, T, N] fp32 buffer that the following row kernel reduces in a fixed order (no float
//     atomics: results are reproducible run to run).
//   - The weight tile is the A operand, the activation tile the B operand, so a lane ends up with
//     4 consecutive output columns of one row: float4 stores, and gate/up pairs for SwiGLU in-lane.
//
// fp32 path: plain LDS-tiled FMA kernel, used by fp32 models (correctness configuration).
#include "sled_internal.h"

namespace {

constexpr int KC = 2;    // k-steps (of 32) per pipeline stage
constexpr int NBUF = 4;  // weight register buffers: the stage in use + 3 stages in flight

template <int MT, int NW, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const bf16_t* __restrict__ Xp, const bf16_t* __restrict__ Wp,
                                                        int NT, int KS, int ks_per_split, int T, int T_pad, int N,
                                                        float* __restrict__ out, bf16_t* __restrict__ out_act,
                                                        int F_act) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t* xs = reinterpret_cast<bf16_t*>(smem);  // [2][MT][KC][512]
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

    // One stage of activations is MT*KC KiB: MT*KC*64 16-byte pieces shared out over 256 threads.
    constexpr int XPIECES = (MT * KC * 64 + 255) / 256;
    bf16x8_t wreg[NBUF][NW][KC];
    uint4 xreg[XPIECES];

    auto load_w = [&](int buf, int stage) {
#pragma unroll
        for (int a = 0; a < NW; a++)
#pragma unroll
            for (int c = 0; c < KC; c++)
                wreg[buf][a][c] = *reinterpret_cast<const bf16x8_t*>(wbase[a] + (size_t)(stage * KC + c) * 512);
    };
    // piece e of a stage: row tile e / (KC*64), then KC*512 contiguous elements of that tile's k range
    auto load_x = [&](int stage) {
#pragma unroll
        for (int i = 0; i < XPIECES; i++) {
            const int e = i * 256 + tid;
            if (MT * KC * 64 % 256 == 0 || e < MT * KC * 64) {
                const int b = e / (KC * 64), r = e - b * (KC * 64);
                xreg[i] = *reinterpret_cast<const uint4*>(Xp + ((size_t)(mt_base + b) * KS + ks_begin + stage * KC) * 512 + r * 8);
            }
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int i = 0; i < XPIECES; i++) {
            const int e = i * 256 + tid;
            if (MT * KC * 64 % 256 == 0 || e < MT * KC * 64)
                *reinterpret_cast<uint4*>(xs + (size_t)buf * (MT * KC * 512) + (size_t)e * 8) = xreg[i];
        }
    };
    auto compute = [&](int xbuf, int wbuf) {
#pragma unroll
        for (int c = 0; c < KC; c++) {
#pragma unroll
            for (int b = 0; b < MT; b++) {
                bf16x8_t xf =
                    *reinterpret_cast<const bf16x8_t*>(xs + ((size_t)((xbuf * MT + b) * KC + c)) * 512 + lane * 8);
#pragma unroll
                for (int a = 0; a < NW; a++)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wreg[wbuf][a][c], xf, acc[a][b], 0, 0, 0);
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
        for (int s0 = 0; s0 < n_stage; s0 += NBUF) {
#pragma unroll
            for (int u = 0; u < NBUF; u++) {
                const int s = s0 + u;
                if (s < n_stage) {
                    // Loads are issued oldest-needed first: the activation loads of the next stage are
                    // waited for at the end of this stage, the weight loads three stages later, so the
                    // wait on the former leaves the latter in flight.
                    if (s + 1 < n_stage) load_x(s + 1);
                    if (s + NBUF - 1 < n_stage) load_w((u + NBUF - 1) % NBUF, s + NBUF - 1);
                    compute(u & 1, u);
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
                    uint32_t pk = (uint32_t)f32_to_bf16(a0) | ((uint32_t)f32_to_bf16(a1) << 16);
                    *reinterpret_cast<uint32_t*>(out_act + frag_offset(tok, f, F_act)) = pk;
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
int launch_bf16(int epi, dim3 grid, size_t lds, hipStream_t st, const bf16_t* X, const bf16_t* W, int NT, int KS,
                int kps, int T, int T_pad, int N, float* out, bf16_t* out_act, int F_act) {
    switch (epi) {
        case SLED_EPI_PARTIAL:
            hipLaunchKernelGGL((gemm_bf16_kernel<MT, NW, SLED_EPI_PARTIAL>), grid, dim3(256), lds, st, X, W, NT, KS, kps, T,
                               T_pad, N, out, out_act, F_act);
            break;
        case SLED_EPI_SWIGLU:
            hipLaunchKernelGGL((gemm_bf16_kernel<MT, NW, SLED_EPI_SWIGLU>), grid, dim3(256), lds, st, X, W, NT, KS, kps, T,
                               T_pad, N, out, out_act, F_act);
            break;
        default:
            hipLaunchKernelGGL((gemm_bf16_kernel<MT, NW, SLED_EPI_STORE>), grid, dim3(256), lds, st, X, W, NT, KS, kps, T,
                               T_pad, N, out, out_act, F_act);
            break;
    }
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

}  // namespace

// Number of K slices for a projection of N columns: enough workgroups to cover the chip a few
// times over, slices a multiple of one pipeline stage.
int sled_gemm_pick_split(const sled_model* m, int T, int N, int K) {
    if (m->s.dtype != SLED_BF16) return 1;
    const int n_wg = (N / 16 + 3) / 4;  // one 16-column tile per wavefront, 4 wavefronts
    const int stages = K / (32 * KC);
    int split = 1;
    while (n_wg * split < 256 && split * 2 <= stages && stages % (split * 2) == 0 && K / (split * 2) >= 512) split *= 2;
    return split;
}

int sled_launch_gemm(const sled_model* m, const void* X, const void* W, int T, int T_pad, int N, int K, int epilogue,
                     int split_k, float* out_f32, void* out_act, int F_act, hipStream_t st) {
    if (m->s.dtype == SLED_BF16) {
        if (N % 16 || K % (32 * KC) || T_pad % 16) SLED_FAIL(SLED_EINVAL, "gemm: unsupported shape N=%d K=%d T_pad=%d", N, K, T_pad);
        const int NT = N / 16, KS = K / 32;
        if (KS % split_k || (KS / split_k) % KC) SLED_FAIL(SLED_EINVAL, "gemm: bad split %d for K=%d", split_k, K);
        const int kps = KS / split_k;
        const int mt_total = T_pad / 16;
        // rows are processed in blocks of at most 8 tiles (128 rows), evenly sized
        const int zb = (mt_total + 7) / 8;
        int MT = (mt_total + zb - 1) / zb;
        const int zblocks = (mt_total + MT - 1) / MT;
        const bool wide = ((NT + 7) / 8) * split_k >= 512;  // enough workgroups even with two tiles per wavefront
        dim3 grid(wide ? (NT + 7) / 8 : (NT + 3) / 4, split_k, zblocks);
        size_t lds = (size_t)2 * MT * KC * 512 * sizeof(bf16_t);
        const bf16_t* Xb = static_cast<const bf16_t*>(X);
        const bf16_t* Wb = static_cast<const bf16_t*>(W);
        bf16_t* oa = static_cast<bf16_t*>(out_act);
#define SLED_GEMM_CASE(M_)                                                                                          \
    case M_:                                                                                                       \
        return wide ? launch_bf16<M_, 2>(epilogue, grid, lds, st, Xb, Wb, NT, KS, kps, T, T_pad, N, out_f32, oa, F_act) \
                    : launch_bf16<M_, 1>(epilogue, grid, lds, st, Xb, Wb, NT, KS, kps, T, T_pad, N, out_f32, oa, F_act);
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
