// Vocab-parallel acceptance (greedy match or speculative sampling, Eq. 1 of Sec. 3.1).
//
// Two kernels per call:
//   accept_row_stats   one pass over all logits: per row (split over a few workgroups when the
//                      batch is small) the maximum, its lowest index, and sum exp((z - max)/tau).
//                      Pure HBM scan: four float4 loads in flight per thread, wavefront reductions.
//   accept_finish      one workgroup per request.  Its first wavefront applies the accept test (or the
//                      argmax comparison) to all of the request's rows at once, one row per lane, and
//                      takes the first failure.  In sampling mode the workgroup then draws the request's
//                      one token by inverse CDF from the residual max(0, p - q) of the rejecting row (or
//                      from p of the bonus row), all in float64 and in a fixed order, so that the chosen
//                      token does not depend on anything beyond ~1e-15 of the total mass.  With draft
//                      distributions given as a few (token, probability) pairs per draft, the residual's
//                      mass per tile follows from the sums of p and one pass over the pairs.
#include "sled_internal.h"

#include <type_traits>

namespace {

struct KPack {
    uint8_t k[1024];
};

struct RowStat {
    double s;   // sum of exp((z - m) / tau) over the segment
    float m;    // maximum over the segment
    int idx;    // lowest index attaining it
};

template <bool SAMPLE>
__device__ inline void stat_merge(float& m, int& idx, double& s, float m2, int i2, double s2, float inv_tau) {
    if (m2 > m || (m2 == m && i2 < idx)) {
        if (SAMPLE) s = (m == -INFINITY ? 0.0 : s * (double)expf((m - m2) * inv_tau)) + s2;
        m = m2;
        idx = i2;
    } else if (SAMPLE) {
        s += (m2 == -INFINITY ? 0.0 : s2 * (double)expf((m2 - m) * inv_tau));
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

    // a chunk of values in ascending index order: its maximum first, then one rescale of the running sum, then
    // the chunk's terms (summed in float32, as accurate as the float32 exponentials themselves)
    auto take = [&](const float* x, const int* vi, auto n_c) {
        constexpr int n = decltype(n_c)::value;
        float cm = x[0];
        int ci = vi[0];
#pragma unroll
        for (int e = 1; e < n; e++)
            if (x[e] > cm) {
                cm = x[e];
                ci = vi[e];
            }
        if (cm > m) {
            if (SAMPLE) s *= (double)expf((m - cm) * inv_tau);  // m = -inf: s is still 0
            m = cm;
            idx = ci;
        }
        if (SAMPLE) {
            float cs = 0.f;
#pragma unroll
            for (int e = 0; e < n; e++) cs += expf((x[e] - m) * inv_tau);  // padding is -inf: adds 0
            s += (double)cs;
        }
    };

    if ((V & 3) == 0 && (reinterpret_cast<uintptr_t>(logits) & 15) == 0) {
        // seg is a multiple of 4 and rows are 16-byte aligned
        const float4* z4 = reinterpret_cast<const float4*>(z);
        const int e4 = v1 / 4;
        for (int v = v0 / 4 + threadIdx.x; v < e4; v += 256 * 4) {
            float4 q[4];
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const int vv = v + 256 * u;
                q[u] = vv < e4 ? z4[vv] : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            }
            float x[16];
            int vi[16];
#pragma unroll
            for (int u = 0; u < 4; u++) {
                x[4 * u] = q[u].x;
                x[4 * u + 1] = q[u].y;
                x[4 * u + 2] = q[u].z;
                x[4 * u + 3] = q[u].w;
#pragma unroll
                for (int e = 0; e < 4; e++) vi[4 * u + e] = 4 * (v + 256 * u) + e;
            }
            take(x, vi, std::integral_constant<int, 16>{});
        }
    } else {
        for (int v = v0 + threadIdx.x; v < v1; v += 256) {
            const float x = z[v];
            take(&x, &v, std::integral_constant<int, 1>{});
        }
    }
    if (idx == 0x7fffffff) {  // this thread saw nothing
        m = -INFINITY;
        s = 0.0;
    }
    // wavefront reduction, then across the 4 wavefronts through LDS
    for (int off = 32; off > 0; off >>= 1) {
        const float m2 = __shfl_xor(m, off);
        const int i2 = __shfl_xor(idx, off);
        const double s2 = __shfl_xor(s, off);
        stat_merge<SAMPLE>(m, idx, s, m2, i2, s2, inv_tau);
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
        for (int i = 1; i < 4; i++) stat_merge<SAMPLE>(m, idx, s, sm[i], si[i], ss[i], inv_tau);
        RowStat r;
        r.s = s;
        r.m = m;
        r.idx = idx;
        stats[(size_t)row * n_split + split] = r;
    }
}

// statistics of a whole row from those of its segments, merged in ascending order
__device__ inline void row_stat(const RowStat* __restrict__ st, int n_split, float inv_tau, float& m, int& amax, double& S) {
    m = st[0].m;
    amax = st[0].idx;
    S = st[0].s;
    for (int sp = 1; sp < n_split; sp++) {
        const float m2 = st[sp].m;
        if (m2 == -INFINITY) continue;
        if (m2 > m) {  // strictly greater: equal maxima keep the lower index (earlier segment)
            S = S * exp(((double)m - (double)m2) * (double)inv_tau) + st[sp].s;
            m = m2;
            amax = st[sp].idx;
        } else {
            S += st[sp].s * exp(((double)m2 - (double)m) * (double)inv_tau);
        }
    }
}

// Where the draft distributions come from: dense rows q[sum k, V], or, per draft, `m` (token id, probability)
// pairs of a distribution that is zero elsewhere (ids distinct; an entry with probability 0 or an id outside
// the vocabulary is padding).
// With `rest` (sparse only): the pairs carry the probabilities as the drafter had them, not renormalised, and
// rest[draft] is the mass of everything not listed, taken to be spread evenly over the unlisted tokens.
struct QSrc {
    const float* dense;
    const int32_t* ids;
    const float* probs;
    const float* rest;
    int m;  // 0: dense
};

__device__ inline bool q_entry_real(int id, float pr, int V) { return id >= 0 && id < V && pr > 0.f; }

// probability of an unlisted token: the remainder mass over the number of unlisted tokens
__device__ inline double q_background(const QSrc& q, int qrow, int V, int n_real) {
    if (!q.rest || n_real >= V) return 0.0;
    return (double)q.rest[qrow] / (double)(V - n_real);
}

__device__ inline double q_of(const QSrc& q, int qrow, int V, int d) {
    if (q.m == 0) return (double)q.dense[(size_t)qrow * V + d];
    double v = 0.0;
    bool found = false;
    int n_real = 0;
    for (int i = 0; i < q.m; i++) {
        const int id = q.ids[(size_t)qrow * q.m + i];
        const float pr = q.probs[(size_t)qrow * q.m + i];
        if (!q_entry_real(id, pr, V)) continue;
        n_real++;
        if (id == d) {
            v = (double)pr;
            found = true;
        }
    }
    return found ? v : q_background(q, qrow, V, n_real);
}

struct Decision {
    int a;       // accepted prefix length
    int row;     // packed row the output token comes from (row0 + a)
    int qrow;    // draft row whose q is subtracted there, or -1 (all accepted: bonus row)
    float m;     // that row's maximum
    int amax;    // and its argmax
};

// One wavefront decides one request: lane j judges draft j+1 against row j; the first failing lane ends the
// accepted prefix (Eq. 1; in greedy mode the test is equality with the row's argmax).
__device__ inline Decision decide_request(int mode, int i, const KPack& kp, int V, int n_split, float inv_tau, double it,
                                          const float* __restrict__ logits, const int32_t* __restrict__ tokens,
                                          const QSrc& draft_q, const float* __restrict__ u_acc,
                                          const RowStat* __restrict__ stats, int lane) {
    int row0 = 0;
    for (int r = lane; r < i; r += 64) row0 += kp.k[r];
    for (int off = 32; off > 0; off >>= 1) row0 += __shfl_xor(row0, off);
    const int d0 = row0;   // drafts before this request
    row0 += i;             // rows before it: one more per request
    const int k = kp.k[i];
    int a = k;
    for (int j0 = 0; j0 < k; j0 += 64) {
        const int j = j0 + lane;
        bool fail = false, close = false;
        float m = 0.f;
        double zd = 0.0, lhs = 0.0;
        if (j < k) {
            int amax;
            double S;
            row_stat(stats + (size_t)(row0 + j) * n_split, n_split, inv_tau, m, amax, S);
            const int d = tokens[row0 + j + 1];
            if (mode == SLED_GREEDY) {
                fail = (d != amax);
            } else if (d < 0 || d >= V) {
                fail = true;  // a draft outside the vocabulary has no target probability: rejected where it stands
            } else {
                zd = (double)logits[(size_t)(row0 + j) * V + d];
                const double pd = exp((zd - (double)m) * it) / S;
                lhs = (double)u_acc[d0 + j] * q_of(draft_q, d0 + j, V, d);
                fail = !(lhs <= pd);
                // S carries the float32 round-off of the row scan (about 1e-7): a test this close is decided again below
                close = fabs(lhs - pd) <= 1e-4 * pd;
            }
        }
        // Rare: the two sides of Eq. 1 agree to four digits.  The whole wavefront then sums the row's normaliser in
        // float64, in a fixed order (lane-strided partial sums, then a butterfly), and the lane decides again.
        unsigned long long todo = __ballot(close);
        while (todo) {
            const int src = __ffsll((long long)todo) - 1;
            todo &= todo - 1;
            const float ms = __shfl(m, src);
            const float* z = logits + (size_t)(row0 + j0 + src) * V;
            double part = 0.0;
            for (int v = lane; v < V; v += 64) part += exp(((double)z[v] - (double)ms) * it);
            for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
            if (lane == src) fail = !(lhs <= exp((zd - (double)m) * it) / part);
        }
        const unsigned long long mask = __ballot(fail);
        if (mask) {
            a = j0 + __ffsll((long long)mask) - 1;
            break;
        }
    }
    Decision dc;
    dc.a = a;
    dc.row = row0 + a;
    dc.qrow = a < k ? d0 + a : -1;
    double S;
    row_stat(stats + (size_t)dc.row * n_split, n_split, inv_tau, dc.m, dc.amax, S);
    return dc;
}

constexpr int SLED_SPARSE_Q_MAX = 1024;  // entries per draft of a sparse draft distribution
constexpr int WTILE = 1024;        // elements per wavefront tile: 16 consecutive ones per lane
constexpr int MAX_WTILES = 2048;   // covers vocabularies up to 2 097 152

__global__ __launch_bounds__(1024) void accept_finish(int mode, KPack kp, int V, int n_split, float inv_tau, float temperature,
                                                      const float* __restrict__ logits, const int32_t* __restrict__ tokens,
                                                      QSrc qsrc, const float* __restrict__ u_acc,
                                                      const float* __restrict__ u_smp, const RowStat* __restrict__ stats,
                                                      int32_t* __restrict__ accept_len, int32_t* __restrict__ out_token) {
    __shared__ double tile_sum[MAX_WTILES];
    __shared__ double sp_take[SLED_SPARSE_Q_MAX];   // sparse q: probability mass entry i removes from p
    __shared__ int sp_tile[SLED_SPARSE_Q_MAX];      //           and the tile it falls in (-1: padding)
    __shared__ double q_tile[WTILE];                //           q over the tile that holds the draw
    __shared__ Decision sh_dc;
    __shared__ int sh_tile, sh_real;
    __shared__ double sh_base, sh_total;
    const int i = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, n_wv = blockDim.x >> 6;
    if (wv == 0) {
        // float64 work divides by the temperature as given (a float32 number), exactly as a float64 reference does
        const Decision dc = decide_request(mode, i, kp, V, n_split, inv_tau, 1.0 / (double)temperature, logits, tokens, qsrc, u_acc, stats, lane);
        if (lane == 0) {
            sh_dc = dc;
            accept_len[i] = dc.a;
            if (mode == SLED_GREEDY) out_token[i] = dc.amax;
        }
    }
    if (mode == SLED_GREEDY) return;
    __syncthreads();
    const Decision dc = sh_dc;
    const float* z = logits + (size_t)dc.row * V;
    const bool sparse = qsrc.m > 0;
    const bool has_q = dc.qrow >= 0;
    const float* q = (has_q && !sparse) ? qsrc.dense + (size_t)dc.qrow * V : nullptr;
    const double m = (double)dc.m, it = 1.0 / (double)temperature;
    const int n_tiles = (V + WTILE - 1) / WTILE;  // at most MAX_WTILES: the host rejects larger vocabularies
    const bool vec = (V & 3) == 0 && (reinterpret_cast<uintptr_t>(logits) & 15) == 0 &&
                     (reinterpret_cast<uintptr_t>(qsrc.dense) & 15) == 0;

    // 16 consecutive values of a row starting at v (0 beyond the end of the row when `pad0`, else -inf)
    auto load16 = [&](const float* p, int v, float* x, float pad) {
        if (vec) {
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const int vv = v + 4 * u;
                float4 t = make_float4(pad, pad, pad, pad);
                if (vv < V) t = *reinterpret_cast<const float4*>(p + vv);
                x[4 * u] = t.x;
                x[4 * u + 1] = t.y;
                x[4 * u + 2] = t.z;
                x[4 * u + 3] = t.w;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 16; e++) x[e] = (v + e < V) ? p[v + e] : pad;
        }
    };
    // this lane's 16 weights of tile t: exp((z - m)/tau) (proportional to p), or max(0, p - q) with p = that / S
    // (with sparse q the residual is only ever needed inside the tile that holds the draw, whose q is in q_tile)
    // (qconst >= 0: the residual against the same q everywhere -- the background of a sparse q with remainder mass)
    auto weights = [&](int t, bool residual, double inv_S, double* w, double qconst = -1.0) {
        const int v = t * WTILE + lane * 16;
        float zx[16], qx[16];
        load16(z, v, zx, -INFINITY);
        if (residual && !sparse) load16(q, v, qx, 0.f);
#pragma unroll
        for (int e = 0; e < 16; e++) {
            const double ev = exp(((double)zx[e] - m) * it);  // exp(-inf) = 0 beyond the row
            if (residual) {
                const double r = ev * inv_S - (qconst >= 0.0 ? qconst : sparse ? q_tile[lane * 16 + e] : (double)qx[e]);
                w[e] = r > 0.0 ? r : 0.0;
            } else {
                w[e] = ev;
            }
        }
    };
    // every wavefront sums whole tiles (lane order, then a butterfly): no workgroup barrier per tile
    auto sweep = [&](bool residual, double inv_S, double qconst = -1.0) {
        for (int t = wv; t < n_tiles; t += n_wv) {
            double w[16];
            weights(t, residual, inv_S, w, qconst);
            double acc = 0.0;
#pragma unroll
            for (int e = 0; e < 16; e++) acc += w[e];
            for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
            if (lane == 0) tile_sum[t] = acc;
        }
        __syncthreads();
    };
    // wavefront 0: total of the tile sums (ascending), the tile in which the running sum first exceeds
    // u * total, and the running sum before that tile
    auto locate = [&](double u) {
        if (wv == 0) {
            const int per = (n_tiles + 63) / 64;
            const int t0 = lane * per, t1 = min(n_tiles, t0 + per);
            double part = 0.0;
            for (int t = t0; t < t1; t++) part += tile_sum[t];
            double incl = part;
            for (int off = 1; off < 64; off <<= 1) {
                const double o = __shfl_up(incl, off);
                if (lane >= off) incl += o;
            }
            const double total = __shfl(incl, 63);
            const double target = u * total;
            const unsigned long long mask = __ballot(incl > target && t1 > t0);
            // round-off can leave no lane past the target: then the last tile holds the crossing
            const int owner = mask ? __ffsll((long long)mask) - 1 : (n_tiles - 1) / per;
            if (lane == owner) {
                double c = incl - part;
                int tt = t1 - 1;
                for (int t = t0; t < t1; t++) {
                    if (c + tile_sum[t] > target) {
                        tt = t;
                        break;
                    }
                    if (t < t1 - 1) c += tile_sum[t];
                }
                sh_tile = tt;
                sh_base = c;
                sh_total = total;
            }
        }
        __syncthreads();
    };

    const double u = (double)u_smp[i];
    double qbg = 0.0;   // sparse q with remainder mass: probability of a token that is not listed
    bool residual = false;
    double inv_S = 1.0;
    sweep(false, 1.0);  // tile sums of exp((z - m)/tau); their total is the normaliser S
    locate(u);
    if (has_q) {
        const double S = sh_total;
        __syncthreads();  // everybody has read the total before the tile sums are replaced
        if (!sparse) {
            sweep(true, 1.0 / S);
        } else {
            // sum over a tile of max(0, p - q) = background - sum over the entries in it of what listing them takes
            // away, where the background is the tile's residual against the probability c of an unlisted token.
            // Without remainder mass c = 0: the background is the sum of p, known from the first sweep, and an entry
            // takes min(p, q) -- one pass over the m entries instead of a second pass over the vocabulary.  With
            // remainder mass the background needs that second pass (against the constant c), and an entry takes
            // max(0, p - c) - max(0, p - q).
            const int32_t* ids = qsrc.ids + (size_t)dc.qrow * qsrc.m;
            const float* pr = qsrc.probs + (size_t)dc.qrow * qsrc.m;
            if (tid == 0) {
                int n_real = 0;
                for (int e = 0; e < qsrc.m; e++) n_real += q_entry_real(ids[e], pr[e], V);
                sh_real = n_real;
            }
            __syncthreads();
            qbg = q_background(qsrc, dc.qrow, V, sh_real);
            if (qbg > 0.0) {
                sweep(true, 1.0 / S, qbg);
            }
            for (int e = tid; e < qsrc.m; e += blockDim.x) {
                const int id = ids[e];
                const double qv = (double)pr[e];
                const bool real = q_entry_real(id, pr[e], V);
                double take = 0.0;
                if (real) {
                    const double pv = exp(((double)z[id] - m) * it) * (1.0 / S);
                    const double with_c = pv > qbg ? pv - qbg : 0.0, with_q = pv > qv ? pv - qv : 0.0;
                    take = with_c - with_q;
                }
                sp_take[e] = take;
                sp_tile[e] = real ? id / WTILE : -1;
            }
            __syncthreads();
            for (int t = tid; t < n_tiles; t += blockDim.x) {
                double r = qbg > 0.0 ? tile_sum[t] : tile_sum[t] * (1.0 / S);
                for (int e = 0; e < qsrc.m; e++)   // in entry order: the result does not depend on the thread layout
                    if (sp_tile[e] == t) r -= sp_take[e];
                tile_sum[t] = r > 0.0 ? r : 0.0;
            }
            __syncthreads();
        }
        locate(u);
        if (sh_total > 0.0) {
            residual = true;
            inv_S = 1.0 / S;
        } else {
            // the residual has no mass (p <= q everywhere up to round-off): draw from p instead
            __syncthreads();
            sweep(false, 1.0);
            locate(u);
        }
    }
    if (residual && sparse) {
        // q over the tile of the draw, dense in LDS
        const int tt0 = sh_tile;
        for (int e = tid; e < WTILE; e += blockDim.x) q_tile[e] = qbg;
        __syncthreads();
        const int32_t* ids = qsrc.ids + (size_t)dc.qrow * qsrc.m;
        const float* pr = qsrc.probs + (size_t)dc.qrow * qsrc.m;
        for (int e = tid; e < qsrc.m; e += blockDim.x)
            if (sp_tile[e] == tt0) q_tile[ids[e] - tt0 * WTILE] = (double)pr[e];   // (ids are distinct within a row)
        __syncthreads();
    }
    if (wv != 0) return;
    // inside the tile: 16 weights per lane, an ordered scan over the lanes, then over the lane's own 16
    const int tt = sh_tile;
    const double target = u * sh_total;
    double w[16];
    weights(tt, residual, inv_S, w);
    double part = 0.0;
#pragma unroll
    for (int e = 0; e < 16; e++) part += w[e];
    double incl = part;
    for (int off = 1; off < 64; off <<= 1) {
        const double o = __shfl_up(incl, off);
        if (lane >= off) incl += o;
    }
    const unsigned long long cross = __ballot(sh_base + incl > target);
    int found = -1;
    if (cross) {
        const int owner = __ffsll((long long)cross) - 1;
        if (lane == owner) {
            double c = sh_base + (incl - part);
            for (int e = 0; e < 16 && found < 0; e++) {
                if (c + w[e] > target) found = tt * WTILE + lane * 16 + e;
                else c += w[e];
            }
        }
        found = __shfl(found, owner);
    }
    if (found < 0) {
        // round-off between the two summation orders hid the crossing: the last index of the tile that carries
        // weight (of the row, if the tile carries none)
        int last = -1;
        for (int e = 15; e >= 0; e--)
            if (w[e] > 0.0) {
                last = tt * WTILE + lane * 16 + e;
                break;
            }
        for (int off = 32; off > 0; off >>= 1) last = max(last, __shfl_xor(last, off));
        found = last >= 0 ? last : dc.amax;
    }
    if (lane == 0) out_token[i] = found;
}

// confidence of every row: 1 / sum exp((z - max) / tau) is the probability of the most likely token
__global__ void row_confidence_finish(const RowStat* __restrict__ stats, int T, int n_split, float inv_tau,
                                      float* __restrict__ conf, int32_t* __restrict__ top) {
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= T) return;
    float m = -INFINITY;
    int idx = 0x7fffffff;
    double s = 0.0;
    for (int sp = 0; sp < n_split; sp++) {  // segments in ascending order of token id
        const RowStat r = stats[(size_t)row * n_split + sp];
        stat_merge<true>(m, idx, s, r.m, r.idx, r.s, inv_tau);
    }
    conf[row] = (float)(1.0 / s);
    if (top) top[row] = idx;
}

}  // namespace

size_t sled_accept_ws_bytes(int B, int T, int n_split) {
    (void)B;
    size_t stats = (size_t)T * n_split * sizeof(RowStat);
    return (stats + 255) & ~(size_t)255;
}

int sled_accept_pick_split(int T, int vocab) {
    // enough workgroups (rows x segments) for several rounds over the chip, so that the last round is short
    int n = (8192 + T - 1) / T;
    if (n > 16) n = 16;
    if (n < 1) n = 1;
    while (n > 1 && vocab / n < 2048) n--;
    return n;
}

int sled_launch_accept(int mode, int B, int T, const int* k_host, int vocab, float temperature, const float* logits,
                       const int32_t* tokens, const float* draft_q, const int32_t* q_ids, const float* q_probs,
                       const float* q_rest, int q_m, const float* u_acc, const float* u_smp, int32_t* accept_len, int32_t* out_token, void* ws,
                       hipStream_t st) {
    if ((vocab + WTILE - 1) / WTILE > MAX_WTILES) SLED_FAIL(SLED_EINVAL, "accept: vocabulary %d too large", vocab);
    if (q_m < 0 || q_m > SLED_SPARSE_Q_MAX) SLED_FAIL(SLED_EINVAL, "accept: %d sparse entries per draft, at most %d", q_m, SLED_SPARSE_Q_MAX);
    KPack kp;
    for (int i = 0; i < B; i++) kp.k[i] = (uint8_t)k_host[i];
    QSrc qsrc{draft_q, q_ids, q_probs, q_m > 0 ? q_rest : nullptr, q_m};
    const int n_split = sled_accept_pick_split(T, vocab);
    int seg = (vocab + n_split - 1) / n_split;
    seg = (seg + 3) & ~3;
    RowStat* stats = reinterpret_cast<RowStat*>(ws);
    const float inv_tau = 1.0f / temperature;
    dim3 grid(T, n_split);
    if (mode == SLED_SAMPLE)
        hipLaunchKernelGGL(accept_row_stats<true>, grid, dim3(256), 0, st, logits, vocab, n_split, seg, inv_tau, stats);
    else
        hipLaunchKernelGGL(accept_row_stats<false>, grid, dim3(256), 0, st, logits, vocab, n_split, seg, inv_tau, stats);
    SLED_LAUNCH_CHECK();
    // greedy needs only the deciding wavefront
    hipLaunchKernelGGL(accept_finish, dim3(B), dim3(mode == SLED_SAMPLE ? 1024 : 64), 0, st, mode, kp, vocab, n_split, inv_tau,
                       temperature, logits, tokens, qsrc, u_acc, u_smp, stats, accept_len, out_token);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

// ---------------------------------------------------------------------------------------------------------------
// sled_accept for callers that cannot allocate: the row statistics live in a fixed array of device memory that is
// part of the library's code object (one copy per GPU, held until the process ends) instead of a caller's workspace.
constexpr size_t SLED_STATIC_STATS = 16384;   // row-segment statistics: 256 KiB
static __device__ __align__(256) unsigned char scratch[SLED_STATIC_STATS * sizeof(RowStat)];

namespace {
constexpr int SLED_MAX_DEVICES = 64;
void* g_scratch_ptr[SLED_MAX_DEVICES];   // device address of `scratch` on each GPU (the array's name is no address on the host)

// the address of this GPU's copy of the array, looked up once per device with that device current
int static_scratch(void** out) {
    int dev = -1;
    SLED_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= SLED_MAX_DEVICES) SLED_FAIL(SLED_EINVAL, "sled_accept_static: device %d unsupported", dev);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        SLED_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) SLED_FAIL(SLED_EHIP, "sled_accept_static: no device address for the static scratch array");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SLED_OK;
}
}  // namespace

extern "C" int sled_accept_static(int mode, int B, const int* k, int vocab, float temperature, const float* logits,
                                  const int32_t* tokens, const float* draft_q, const float* u_acc, const float* u_smp,
                                  int32_t* accept_len, int32_t* out_token, void* stream) {
    if (!k || !logits || !tokens || !accept_len || !out_token) SLED_FAIL(SLED_EINVAL, "sled_accept_static: null argument");
    if (mode != SLED_GREEDY && mode != SLED_SAMPLE) SLED_FAIL(SLED_EINVAL, "sled_accept_static: unknown mode %d", mode);
    if (B < 1 || B > 1024) SLED_FAIL(SLED_EINVAL, "sled_accept_static: batch size %d outside [1, 1024]", B);
    if (vocab < 2 || vocab > 2000000) SLED_FAIL(SLED_EINVAL, "sled_accept_static: vocab %d unsupported", vocab);
    if (!(temperature > 0.f)) SLED_FAIL(SLED_EINVAL, "sled_accept_static: temperature must be positive");
    int T = 0, nd = 0;
    for (int i = 0; i < B; i++) {
        if (k[i] < 0 || k[i] > 255) SLED_FAIL(SLED_EINVAL, "sled_accept_static: k[%d] = %d outside [0, 255]", i, k[i]);
        T += k[i] + 1;
        nd += k[i];
    }
    if (mode == SLED_SAMPLE && (!u_smp || (nd > 0 && (!draft_q || !u_acc))))
        SLED_FAIL(SLED_EINVAL, "sled_accept_static: sampling needs draft_q, u_acc and u_smp");
    const size_t need = (size_t)T * sled_accept_pick_split(T, vocab);
    if (need > SLED_STATIC_STATS)
        SLED_FAIL(SLED_EINVAL, "sled_accept_static: %d rows in %d segments need %zu statistics, the static scratch holds %zu; use sled_accept",
                  T, sled_accept_pick_split(T, vocab), need, SLED_STATIC_STATS);
    void* ws = nullptr;
    int rc = static_scratch(&ws);
    if (rc != SLED_OK) return rc;
    // nothing in the array has to start at zero: the row scan writes every statistic the finish kernel reads
    return sled_launch_accept(mode, B, T, k, vocab, temperature, logits, tokens, draft_q, nullptr, nullptr, nullptr, 0, u_acc,
                              u_smp, accept_len, out_token, ws, static_cast<hipStream_t>(stream));
}

int sled_launch_row_confidence(int T, int vocab, float temperature, const float* logits, float* conf, int32_t* top, void* ws,
                               hipStream_t st) {
    const int n_split = sled_accept_pick_split(T, vocab);
    int seg = (vocab + n_split - 1) / n_split;
    seg = (seg + 3) & ~3;
    RowStat* stats = reinterpret_cast<RowStat*>(ws);
    const float inv_tau = 1.0f / temperature;
    hipLaunchKernelGGL(accept_row_stats<true>, dim3(T, n_split), dim3(256), 0, st, logits, vocab, n_split, seg, inv_tau, stats);
    SLED_LAUNCH_CHECK();
    hipLaunchKernelGGL(row_confidence_finish, dim3((T + 255) / 256), dim3(256), 0, st, stats, T, n_split, inv_tau, conf, top);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}
