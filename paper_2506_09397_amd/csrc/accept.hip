// Vocab-parallel acceptance (greedy match or speculative sampling, Eq. 1 of Sec. 3.1).
//
// Three kernels:
//   accept_row_stats   one pass over all logits: per row (split over a few workgroups when the
//                      batch is small) the maximum, its lowest index, and sum exp((z - max)/tau).
//                      Pure HBM scan: float4 loads, wavefront reductions.
//   accept_decide      one thread per request: walks the request's rows in order, applies the
//                      accept test (or the argmax comparison) and records where it stopped.
//   accept_resample    sampling only, one workgroup per request: inverse-CDF draw from the
//                      residual max(0, p - q) of the rejecting row (or from p of the bonus row),
//                      all in float64 so that the chosen token does not depend on summation order
//                      beyond ~1e-15 of the total mass.
#include "sled_internal.h"

namespace {

struct KPack {
    uint8_t k[1024];
};

struct RowStat {
    double s;   // sum of exp((z - m) / tau) over the segment
    float m;    // maximum over the segment
    int idx;    // lowest index attaining it
};

struct ReqPlan {      // written by accept_decide, read by accept_resample
    int row;          // packed row to draw from
    int qrow;         // draft row whose q is subtracted, or -1 (bonus draw from p)
    float m;          // that row's maximum
};

__device__ inline void stat_merge(float& m, int& idx, double& s, float m2, int idx2, double s2, float inv_tau) {
    if (m2 > m || (m2 == m && idx2 < idx)) {
        // rescale our sum to the new maximum
        s = s * (double)__expf((m - m2) * inv_tau) + s2;
        if (m2 == m) s = s;  // equal maxima: factor is exactly 1
        m = m2;
        idx = idx2;
    } else {
        s = s + s2 * (double)__expf((m2 - m) * inv_tau);
    }
}

template <bool SAMPLE>
__global__ __launch_bounds__(256) void accept_row_stats(const float* __restrict__ logits, int V, int n_split, int seg,
                                                        float inv_tau, RowStat* __restrict__ stats) {
    const int row = blockIdx.x, split = blockIdx.y;
    const int v0 = split * seg;
    const int v1 = min(V, v0 + seg);
    const float* z = logits + (size_t)row * V;
    float m = -INFINITY;
    int idx = 0x7fffffff;
    double s = 0.0;

    auto take = [&](float x, int v) {
        if (x > m) {
            if (SAMPLE) s = s * (double)expf((m - x) * inv_tau) + 1.0;
            m = x;
            idx = v;
        } else if (SAMPLE) {
            s += (double)expf((x - m) * inv_tau);
        }
    };

    if ((V & 3) == 0) {
        // seg is a multiple of 4 and rows are 16-byte aligned
        const float4* z4 = reinterpret_cast<const float4*>(z);
        for (int v = v0 / 4 + threadIdx.x; v < v1 / 4; v += 256) {
            float4 x = z4[v];
            take(x.x, 4 * v);
            take(x.y, 4 * v + 1);
            take(x.z, 4 * v + 2);
            take(x.w, 4 * v + 3);
        }
    } else {
        for (int v = v0 + threadIdx.x; v < v1; v += 256) take(z[v], v);
    }
    if (idx == 0x7fffffff) {  // this thread saw nothing
        m = -INFINITY;
        s = 0.0;
    }
    // wavefront reduction, then across the 4 wavefronts through LDS
    for (int off = 32; off > 0; off >>= 1) {
        float m2 = __shfl_xor(m, off);
        int i2 = __shfl_xor(idx, off);
        double s2 = __shfl_xor(s, off);
        if (m2 > m || (m2 == m && i2 < idx)) {
            if (SAMPLE) s = (m == -INFINITY ? 0.0 : s * (double)expf((m - m2) * inv_tau)) + s2;
            m = m2;
            idx = i2;
        } else if (SAMPLE) {
            s += (m2 == -INFINITY ? 0.0 : s2 * (double)expf((m2 - m) * inv_tau));
        }
    }
    __shared__ float sm[4];
    __shared__ int si[4];
    __shared__ double ss[4];
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
        sm[w] = m;
        si[w] = idx;
        ss[w] = s;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < 4; i++) {
            float m2 = sm[i];
            int i2 = si[i];
            double s2 = ss[i];
            if (m2 > m || (m2 == m && i2 < idx)) {
                if (SAMPLE) s = (m == -INFINITY ? 0.0 : s * (double)expf((m - m2) * inv_tau)) + s2;
                m = m2;
                idx = i2;
            } else if (SAMPLE) {
                s += (m2 == -INFINITY ? 0.0 : s2 * (double)expf((m2 - m) * inv_tau));
            }
        }
        RowStat r;
        r.s = s;
        r.m = m;
        r.idx = idx;
        stats[(size_t)row * n_split + split] = r;
    }
}

__global__ void accept_decide(int mode, int B, KPack kp, int V, int n_split, float inv_tau,
                              const float* __restrict__ logits, const int32_t* __restrict__ tokens,
                              const float* __restrict__ draft_q, const float* __restrict__ u_acc,
                              const RowStat* __restrict__ stats, int32_t* __restrict__ accept_len,
                              int32_t* __restrict__ out_token, ReqPlan* __restrict__ plan) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B) return;
    int row0 = 0, d0 = 0;
    for (int r = 0; r < i; r++) {
        row0 += kp.k[r] + 1;
        d0 += kp.k[r];
    }
    const int k = kp.k[i];
    int a = 0;
    float m = 0.f;
    int amax = 0;
    double S = 0.0;
    for (int j = 0; j <= k; j++) {
        // merge the row's segments in ascending order
        const RowStat* st = stats + (size_t)(row0 + j) * n_split;
        m = st[0].m;
        amax = st[0].idx;
        S = st[0].s;
        for (int sp = 1; sp < n_split; sp++) {
            float m2 = st[sp].m;
            if (m2 == -INFINITY) continue;
            if (m2 > m) {  // strictly greater: equal maxima keep the lower index (earlier segment)
                S = S * exp(((double)m - (double)m2) * (double)inv_tau) + st[sp].s;
                m = m2;
                amax = st[sp].idx;
            } else {
                S += st[sp].s * exp(((double)m2 - (double)m) * (double)inv_tau);
            }
        }
        if (j == k) break;  // bonus row: nothing left to judge
        const int d = tokens[row0 + j + 1];
        bool ok;
        if (mode == SLED_GREEDY) {
            ok = (d == amax);
        } else {
            const double zd = (double)logits[(size_t)(row0 + j) * V + d];
            const double pd = exp((zd - (double)m) * (double)inv_tau) / S;
            const double lhs = (double)u_acc[d0 + j] * (double)draft_q[(size_t)(d0 + j) * V + d];
            ok = (lhs <= pd);
        }
        if (!ok) break;
        a = j + 1;
    }
    accept_len[i] = a;
    if (mode == SLED_GREEDY) {
        out_token[i] = amax;
    } else {
        ReqPlan pl;
        pl.row = row0 + a;
        pl.qrow = (a < k) ? (d0 + a) : -1;
        pl.m = m;
        plan[i] = pl;
    }
}

// block-wide sum of doubles over 1024 threads; every thread gets the result
__device__ inline double block_sum_1024(double x, double* sh /*[16]*/) {
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = x;
    __syncthreads();
    double t = 0.0;
    for (int i = 0; i < 16; i++) t += sh[i];
    return t;
}

__global__ __launch_bounds__(1024) void accept_resample(int V, float inv_tau, const float* __restrict__ logits,
                                                        const float* __restrict__ draft_q,
                                                        const float* __restrict__ u_smp,
                                                        const ReqPlan* __restrict__ plan,
                                                        int32_t* __restrict__ out_token) {
    __shared__ double sh[16];
    __shared__ double tile_sum[512];
    __shared__ double thread_sum[1024];
    __shared__ int result;
    const int i = blockIdx.x;
    const ReqPlan pl = plan[i];
    const float* z = logits + (size_t)pl.row * V;
    const float* q = pl.qrow >= 0 ? draft_q + (size_t)pl.qrow * V : nullptr;
    const double m = (double)pl.m, it = (double)inv_tau;
    const int tid = threadIdx.x;

    // sweep A: normaliser of p in float64
    double acc = 0.0;
    for (int v = tid; v < V; v += 1024) acc += exp(((double)z[v] - m) * it);
    const double S = block_sum_1024(acc, sh);

    const int TILE = 4096;  // 4 consecutive elements per thread per tile
    const int n_tiles = (V + TILE - 1) / TILE;
    if (n_tiles > 512) {  // host rejects such vocabularies; never taken
        if (tid == 0) out_token[i] = 0;
        return;
    }
    auto weight = [&](int v, bool use_q) -> double {
        double p = exp(((double)z[v] - m) * it) / S;
        if (use_q) {
            double r = p - (double)q[v];
            return r > 0.0 ? r : 0.0;
        }
        return p;
    };

    bool use_q = (q != nullptr);
    for (int attempt = 0; attempt < 2; attempt++) {
        // sweep B: mass of each tile
        for (int t = 0; t < n_tiles; t++) {
            double w = 0.0;
            const int v = t * TILE + tid * 4;
            for (int e = 0; e < 4; e++)
                if (v + e < V) w += weight(v + e, use_q);
            double ts = block_sum_1024(w, sh);
            if (tid == 0) tile_sum[t] = ts;
        }
        __syncthreads();
        double total = 0.0;
        for (int t = 0; t < n_tiles; t++) total += tile_sum[t];
        if (total > 0.0 || !use_q) {
            const double target = (double)u_smp[i] * total;
            // tile that holds the crossing (ascending order, running base)
            double base = 0.0;
            int tt = n_tiles - 1;
            for (int t = 0; t < n_tiles; t++) {
                if (base + tile_sum[t] > target) {
                    tt = t;
                    break;
                }
                if (t < n_tiles - 1) base += tile_sum[t];
            }
            if (tt == n_tiles - 1) {  // base for the last tile when the loop ran to its end
                base = 0.0;
                for (int t = 0; t < n_tiles - 1; t++) base += tile_sum[t];
            }
            // sweep C: inside that tile
            double w4[4];
            double w = 0.0;
            const int v = tt * TILE + tid * 4;
            for (int e = 0; e < 4; e++) {
                w4[e] = (v + e < V) ? weight(v + e, use_q) : 0.0;
                w += w4[e];
            }
            thread_sum[tid] = w;
            if (tid == 0) result = -1;
            __syncthreads();
            if (tid < 64) {
                // wavefront 0: each lane sums 16 consecutive thread sums, then an ordered scan over lanes
                double part = 0.0;
                for (int e = 0; e < 16; e++) part += thread_sum[tid * 16 + e];
                double incl = part;
                for (int off = 1; off < 64; off <<= 1) {
                    double o = __shfl_up(incl, off);
                    if (tid >= off) incl += o;
                }
                double excl = incl - part;
                // the lane whose span crosses the target
                bool cross = (base + incl > target);
                unsigned long long mask = __ballot(cross);
                int lane = mask ? (__ffsll((long long)mask) - 1) : -1;
                if (tid == lane) {
                    double c = base + excl;
                    int found = -1;
                    for (int e = 0; e < 16 && found < 0; e++) {
                        int th = tid * 16 + e;
                        if (c + thread_sum[th] > target) found = th;
                        else c += thread_sum[th];
                    }
                    if (found < 0) found = tid * 16 + 15;
                    thread_sum[found] = -1.0 - c;  // mark the owning thread, pass its running base
                }
            }
            __syncthreads();
            if (thread_sum[tid] < 0.0) {
                double c = -1.0 - thread_sum[tid];
                int found = -1;
                for (int e = 0; e < 4 && found < 0; e++) {
                    if (c + w4[e] > target) found = v + e;
                    else c += w4[e];
                }
                result = found;  // -1 if round-off hid the crossing
            }
            __syncthreads();
            if (result < 0) {
                // fallback: last index with positive weight in this tile (or any earlier tile)
                // -- reached only through round-off between the two summation orders
                __shared__ int last_pos;
                if (tid == 0) last_pos = -1;
                __syncthreads();
                for (int e = 3; e >= 0; e--)
                    if (v + e < V && w4[e] > 0.0) {
                        atomicMax(&last_pos, v + e);
                        break;
                    }
                __syncthreads();
                if (tid == 0) result = last_pos >= 0 ? last_pos : 0;
                __syncthreads();
            }
            if (tid == 0) out_token[i] = result;
            return;
        }
        use_q = false;  // residual has no mass (p <= q everywhere up to round-off): draw from p
        __syncthreads();
    }
}

}  // namespace

size_t sled_accept_ws_bytes(int B, int T, int n_split) {
    size_t stats = (size_t)T * n_split * sizeof(RowStat);
    size_t plan = (size_t)B * sizeof(ReqPlan);
    return ((stats + 255) & ~(size_t)255) + ((plan + 255) & ~(size_t)255);
}

int sled_accept_pick_split(int T, int vocab) {
    int n = (1024 + T - 1) / T;
    if (n > 16) n = 16;
    if (n < 1) n = 1;
    while (n > 1 && vocab / n < 2048) n--;
    return n;
}

int sled_launch_accept(int mode, int B, int T, const int* k_host, int vocab, float temperature, const float* logits,
                       const int32_t* tokens, const float* draft_q, const float* u_acc, const float* u_smp,
                       int32_t* accept_len, int32_t* out_token, void* ws, hipStream_t st) {
    KPack kp;
    for (int i = 0; i < B; i++) kp.k[i] = (uint8_t)k_host[i];
    const int n_split = sled_accept_pick_split(T, vocab);
    int seg = (vocab + n_split - 1) / n_split;
    seg = (seg + 3) & ~3;
    RowStat* stats = reinterpret_cast<RowStat*>(ws);
    size_t stats_bytes = ((size_t)T * n_split * sizeof(RowStat) + 255) & ~(size_t)255;
    ReqPlan* plan = reinterpret_cast<ReqPlan*>(reinterpret_cast<char*>(ws) + stats_bytes);
    const float inv_tau = 1.0f / temperature;
    dim3 grid(T, n_split);
    if (mode == SLED_SAMPLE)
        hipLaunchKernelGGL(accept_row_stats<true>, grid, dim3(256), 0, st, logits, vocab, n_split, seg, inv_tau, stats);
    else
        hipLaunchKernelGGL(accept_row_stats<false>, grid, dim3(256), 0, st, logits, vocab, n_split, seg, inv_tau, stats);
    SLED_LAUNCH_CHECK();
    hipLaunchKernelGGL(accept_decide, dim3((B + 63) / 64), dim3(64), 0, st, mode, B, kp, vocab, n_split, inv_tau, logits,
                       tokens, draft_q, u_acc, stats, accept_len, out_token, plan);
    SLED_LAUNCH_CHECK();
    if (mode == SLED_SAMPLE) {
        hipLaunchKernelGGL(accept_resample, dim3(B), dim3(1024), 0, st, vocab, inv_tau, logits, draft_q, u_smp, plan,
                           out_token);
        SLED_LAUNCH_CHECK();
    }
    return SLED_OK;
}
