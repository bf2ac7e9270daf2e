// Row-wise operators of the verify step, one workgroup per packed row.  They sit between the
// projections and do everything that is not a contraction: embedding gather, reduction of the
// split-K partial sums (fixed order), residual add, RMSNorm, rotary embedding, the scatter of new
// K/V into the paged cache, SwiGLU for fp32 models, weight repacking at load time.
//
// Activations that feed a bf16 projection are written directly in MFMA operand order
// (frag_offset), so the projection kernels never transpose anything.  Weights are repacked once, at
// load time, into the k-step-major tile order of wfrag_offset.
#include "sled_internal.h"

#include <algorithm>

namespace {

// sum over the workgroup (blockDim.x a multiple of 64, at most 1024); every thread gets the result;
// the order of additions is fixed
__device__ inline float block_sum(float x, float* sh /*[16]*/) {
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = x;
    __syncthreads();
    float t = 0.f;
    const int nw = blockDim.x >> 6;
    for (int i = 0; i < nw; i++) t += sh[i];
    return t;
}

// store 8 consecutive activations of row t starting at column c0; bf16 models keep an activation
// as a bf16 pair hi + lo in two planes of operand-ordered storage, `plane` elements apart
template <bool BF16>
__device__ inline void store_act8(void* X, size_t plane, int t, int c0, int K, const float* v) {
    if (BF16) {
        uint32_t wh[4], wl[4];
        for (int i = 0; i < 4; i++) {
            const bf16_t h0 = f32_to_bf16(v[2 * i]), h1 = f32_to_bf16(v[2 * i + 1]);
            const bf16_t l0 = f32_to_bf16(v[2 * i] - bf16_to_f32(h0)), l1 = f32_to_bf16(v[2 * i + 1] - bf16_to_f32(h1));
            wh[i] = (uint32_t)h0 | ((uint32_t)h1 << 16);
            wl[i] = (uint32_t)l0 | ((uint32_t)l1 << 16);
        }
        bf16_t* p = static_cast<bf16_t*>(X) + frag_offset(t, c0, K);
        *reinterpret_cast<uint4*>(p) = make_uint4(wh[0], wh[1], wh[2], wh[3]);
        *reinterpret_cast<uint4*>(p + plane) = make_uint4(wl[0], wl[1], wl[2], wl[3]);
    } else {
        float* p = static_cast<float*>(X) + (size_t)t * K + c0;
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
}

// h[t,:] = E[token]; X[t,:] = rmsnorm(h) * gain
template <bool BF16>
__global__ __launch_bounds__(256) void embed_norm_kernel(const int32_t* __restrict__ tokens, const void* __restrict__ E,
                                                         int V, int d, float eps, const float* __restrict__ gain,
                                                         float* __restrict__ h, void* __restrict__ X, size_t plane) {
    __shared__ float sh[16];
    const int t = blockIdx.x;
    int tok = tokens[t];
    tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
    float ss = 0.f;
    for (int c = threadIdx.x * 8; c < d; c += 256 * 8) {
        float v[8];
        if (BF16) {
            uint4 raw = *reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(E) + (size_t)tok * d + c);
            const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
            for (int i = 0; i < 4; i++) {
                v[2 * i] = bf16_to_f32((bf16_t)(w[i] & 0xffff));
                v[2 * i + 1] = bf16_to_f32((bf16_t)(w[i] >> 16));
            }
        } else {
            const float* p = static_cast<const float*>(E) + (size_t)tok * d + c;
            for (int i = 0; i < 8; i++) v[i] = p[i];
        }
        for (int i = 0; i < 8; i++) {
            h[(size_t)t * d + c + i] = v[i];
            ss += v[i] * v[i];
        }
    }
    const float tot = block_sum(ss, sh);
    const float r = 1.0f / sqrtf(tot / (float)d + eps);
    for (int c = threadIdx.x * 8; c < d; c += 256 * 8) {
        float v[8];
        for (int i = 0; i < 8; i++) v[i] = h[(size_t)t * d + c + i] * r * gain[c + i];
        store_act8<BF16>(X, plane, t, c, d, v);
    }
}

// a + sum over the K slices s = 0 .. n_split-1 (ascending) of p[s * stride .. + 3].  The loads of up to eight slices
// are issued before the first is used: a row kernel is a chain of round trips to L2, not a stream, and a loop
// that adds slice after slice would pay one round trip per slice.
__device__ inline float4 add_slices4(float4 a, const float* __restrict__ p, size_t stride, int n_split) {
    for (int s0 = 0; s0 < n_split; s0 += 8) {
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; u++)
            v[u] = s0 + u < n_split ? *reinterpret_cast<const float4*>(p + (size_t)(s0 + u) * stride) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < 8; u++) {
            a.x += v[u].x;
            a.y += v[u].y;
            a.z += v[u].z;
            a.w += v[u].w;
        }
    }
    return a;
}

// the same for two single values
__device__ inline void add_slices1x2(float& a, float& b, const float* __restrict__ pa, const float* __restrict__ pb, size_t stride,
                                     int n_split) {
    for (int s0 = 0; s0 < n_split; s0 += 8) {
        float v[8], w[8];
#pragma unroll
        for (int u = 0; u < 8; u++) {
            const bool on = s0 + u < n_split;
            v[u] = on ? pa[(size_t)(s0 + u) * stride] : 0.f;
            w[u] = on ? pb[(size_t)(s0 + u) * stride] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; u++) {
            a += v[u];
            b += w[u];
        }
    }
}

// ... and for one
__device__ inline float add_slices1(float a, const float* __restrict__ p, size_t stride, int n_split) {
    for (int s0 = 0; s0 < n_split; s0 += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) v[u] = s0 + u < n_split ? p[(size_t)(s0 + u) * stride] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; u++) a += v[u];
    }
    return a;
}

// store 4 consecutive activations of row t starting at column c0 (a multiple of 4), as store_act8 does for 8
template <bool BF16>
__device__ inline void store_act4(void* X, size_t plane, int t, int c0, int K, const float4& v) {
    if (BF16) {
        const float f[4] = {v.x, v.y, v.z, v.w};
        uint32_t wh[2], wl[2];
        for (int i = 0; i < 2; i++) {
            const bf16_t h0 = f32_to_bf16(f[2 * i]), h1 = f32_to_bf16(f[2 * i + 1]);
            const bf16_t l0 = f32_to_bf16(f[2 * i] - bf16_to_f32(h0)), l1 = f32_to_bf16(f[2 * i + 1] - bf16_to_f32(h1));
            wh[i] = (uint32_t)h0 | ((uint32_t)h1 << 16);
            wl[i] = (uint32_t)l0 | ((uint32_t)l1 << 16);
        }
        bf16_t* p = static_cast<bf16_t*>(X) + frag_offset(t, c0, K);  // the 8 elements of a k-octet are contiguous
        *reinterpret_cast<uint2*>(p) = make_uint2(wh[0], wh[1]);
        *reinterpret_cast<uint2*>(p + plane) = make_uint2(wl[0], wl[1]);
    } else {
        *reinterpret_cast<float4*>(static_cast<float*>(X) + (size_t)t * K + c0) = v;
    }
}

// h[t,:] += sum_s partial[s][t][:]  (s ascending);  X[t,:] = rmsnorm(h) * gain.  A thread owns 4 consecutive
// columns per trip over the row; rows of up to 8 * blockDim.x columns (two trips) stay in registers between the
// sum of squares and the scaling, longer rows are read back from h.
template <bool BF16>
__global__ __launch_bounds__(1024) void residual_norm_kernel(const float* __restrict__ partial, int n_split, int T_pad,
                                                            int d, float eps, const float* __restrict__ gain,
                                                            float* __restrict__ h, void* __restrict__ X, size_t plane) {
    __shared__ float sh[16];
    const int t = blockIdx.x;
    const size_t stride = (size_t)T_pad * d;
    const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
    float ss = 0.f;
    if (d <= (int)blockDim.x * 8) {
        float4 a[2] = {zero, zero}, g[2] = {zero, zero};
#pragma unroll
        for (int trip = 0; trip < 2; trip++) {
            const int c = (trip * blockDim.x + threadIdx.x) * 4;
            if (c < d) {
                float* hp = h + (size_t)t * d + c;
                g[trip] = *reinterpret_cast<const float4*>(gain + c);
                a[trip] = add_slices4(*reinterpret_cast<const float4*>(hp), partial + (size_t)t * d + c, stride, n_split);
                *reinterpret_cast<float4*>(hp) = a[trip];
                ss += a[trip].x * a[trip].x + a[trip].y * a[trip].y + a[trip].z * a[trip].z + a[trip].w * a[trip].w;
            }
        }
        const float r = 1.0f / sqrtf(block_sum(ss, sh) / (float)d + eps);
#pragma unroll
        for (int trip = 0; trip < 2; trip++) {
            const int c = (trip * blockDim.x + threadIdx.x) * 4;
            if (c < d)
                store_act4<BF16>(X, plane, t, c, d,
                                 make_float4(a[trip].x * r * g[trip].x, a[trip].y * r * g[trip].y, a[trip].z * r * g[trip].z,
                                             a[trip].w * r * g[trip].w));
        }
        return;
    }
    for (int c = threadIdx.x * 4; c < d; c += blockDim.x * 4) {
        float* hp = h + (size_t)t * d + c;
        const float4 a = add_slices4(*reinterpret_cast<const float4*>(hp), partial + (size_t)t * d + c, stride, n_split);
        *reinterpret_cast<float4*>(hp) = a;
        ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
    }
    const float r = 1.0f / sqrtf(block_sum(ss, sh) / (float)d + eps);
    for (int c = threadIdx.x * 4; c < d; c += blockDim.x * 4) {
        const float4 a = *reinterpret_cast<const float4*>(h + (size_t)t * d + c);  // this thread's own stores
        const float4 g = *reinterpret_cast<const float4*>(gain + c);
        store_act4<BF16>(X, plane, t, c, d, make_float4(a.x * r * g.x, a.y * r * g.y, a.z * r * g.z, a.w * r * g.w));
    }
}

// Per packed row, once per step: cos/sin of pos * theta^(-2i/D), evaluated in float64 and stored as float32, and
// where the row's K/V go (16 * page + slot) -- the chain of dependent lookups behind that is then paid once, not
// in every layer's store kernel.
__global__ void rope_table_kernel(sled_step_meta meta, const int32_t* __restrict__ len_dev, int half, double theta,
                                  float2* __restrict__ cs, int32_t* __restrict__ kvslot) {
    const int t = blockIdx.x;
    const int b = meta.row_req[t];
    const int pos = len_dev[meta.req_id[b]] + meta.pos0[b] + meta.row_j[t];
    if (threadIdx.x == 0) kvslot[t] = meta.pages[meta.cu_pages[b] + (pos >> 4)] * 16 + (pos & 15);
    for (int i = threadIdx.x; i < half; i += blockDim.x) {
        double inv = pow(theta, -(double)i / (double)half);
        double ang = (double)pos * inv;
        cs[(size_t)t * half + i] = make_float2((float)cos(ang), (float)sin(ang));
    }
}

// Per attention work item, once per step: everything its workgroup needs to know before it can request its first
// page, gathered into one 48-byte record -- otherwise each of the step's attention launches starts with a chain of
// four dependent look-ups (item -> block -> request -> committed length).
//   [0] block  [1] kv head  [2] first page  [3] pages  [4] L = context length of the block  [5] rows of the block
//   [6] first packed row  [7] first entry of the block's page list  [8], [9] items of this (block, kv head): first, end
__global__ void attn_plan_kernel(sled_step_meta meta, const int32_t* __restrict__ len_dev, int Hkv, int32_t* __restrict__ plan) {
    const int w = blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= meta.n_work) return;
    const int b = meta.work[4 * w + 0], g = meta.work[4 * w + 1];
    int32_t* r = plan + 12 * w;
    r[0] = b;
    r[1] = g;
    r[2] = meta.work[4 * w + 2];
    r[3] = meta.work[4 * w + 3];
    r[4] = len_dev[meta.req_id[b]] + meta.pos0[b];
    r[5] = meta.k[b] + 1;
    r[6] = meta.cu_rows[b];
    r[7] = meta.cu_pages[b];
    r[8] = meta.cu_work[2 * (b * Hkv + g)];
    r[9] = meta.cu_work[2 * (b * Hkv + g) + 1];
    r[10] = r[11] = 0;
}

// Reduce the QKV partial sums of one head of row t (blockIdx = (t, head), heads ordered q, k, v),
// rotate q and k, write q to Q[T, Hq, D] and k, v into the request's page slot for position L + j.
template <bool BF16>
__global__ __launch_bounds__(64) void qkv_rope_store_kernel(const float* __restrict__ partial, int n_split, int T_pad,
                                                            int Hq, int Hkv, int D, const float2* __restrict__ cs,
                                                            const int32_t* __restrict__ kvslot, void* __restrict__ Q, size_t q_plane, void* __restrict__ k_pool,
                                                            void* __restrict__ v_pool, int64_t n_pages, int layer) {
    const int t = blockIdx.x, head = blockIdx.y;
    const int half = D >> 1;
    const int n_qkv = (Hq + 2 * Hkv) * D;
    const size_t head_elems = (size_t)16 * D;
    const float* prow = partial + (size_t)t * n_qkv;
    const size_t stride = (size_t)T_pad * n_qkv;
    const int ps = kvslot[t], page = ps >> 4, slot = ps & 15;
    if (head < Hq + Hkv) {
        for (int i = threadIdx.x; i < half; i += 64) {
            const int c1 = head * D + i, c2 = c1 + half;
            const float2 sc = cs[(size_t)t * half + i];
            float x1 = 0.f, x2 = 0.f;
            add_slices1x2(x1, x2, prow + c1, prow + c2, stride, n_split);
            float y1, y2;
            rope_pair(x1, x2, sc.x, sc.y, y1, y2);
            if (head < Hq) {
                if (BF16) {  // q is kept as a bf16 pair, like every activation that is not cached
                    bf16_t* q = static_cast<bf16_t*>(Q) + ((size_t)t * Hq + head) * D;
                    const bf16_t h1 = f32_to_bf16(y1), h2 = f32_to_bf16(y2);
                    q[i] = h1;
                    q[i + half] = h2;
                    q[q_plane + i] = f32_to_bf16(y1 - bf16_to_f32(h1));
                    q[q_plane + i + half] = f32_to_bf16(y2 - bf16_to_f32(h2));
                } else {
                    float* q = static_cast<float*>(Q) + ((size_t)t * Hq + head) * D;
                    q[i] = y1;
                    q[i + half] = y2;
                }
            } else {
                const int g = head - Hq;
                const size_t base = (((size_t)layer * n_pages + page) * Hkv + g) * head_elems;
                if (BF16) {
                    // K page-head block in operand order
                    bf16_t* kp = static_cast<bf16_t*>(k_pool) + base;
                    kp[kpage_offset(slot, i)] = f32_to_bf16(y1);
                    kp[kpage_offset(slot, i + half)] = f32_to_bf16(y2);
                } else {
                    float* kp = static_cast<float*>(k_pool) + base + (size_t)slot * D;
                    kp[i] = y1;
                    kp[i + half] = y2;
                }
            }
        }
    } else {
        // v head: no rotation
        const int g = head - Hq - Hkv;
        for (int dd = threadIdx.x; dd < D; dd += 64) {
            const float v = add_slices1(0.f, prow + (Hq + Hkv) * D + g * D + dd, stride, n_split);
            const size_t base = (((size_t)layer * n_pages + page) * Hkv + g) * head_elems;
            if (BF16) {
                static_cast<bf16_t*>(v_pool)[base + vpage_offset(slot, dd)] = f32_to_bf16(v);
            } else {
                static_cast<float*>(v_pool)[base + (size_t)slot * D + dd] = v;
            }
        }
    }
}

// a[t, f] = silu(g) * u with (g, u) = sum over K slices of gu[s][t][2f], gu[s][t][2f+1]; used when the
// gate/up projection does not apply SwiGLU itself (fp32 models, or a gate/up projection split over K).
// One workgroup per row, 8 outputs per thread.
template <bool BF16>
__global__ __launch_bounds__(256) void swiglu_reduce_kernel(const float* __restrict__ gu, int n_split, int T_pad, int F,
                                                            void* __restrict__ A, size_t plane) {
    const int t = blockIdx.x;
    for (int f0 = (blockIdx.y * 256 + threadIdx.x) * 8; f0 < F; f0 += gridDim.y * 256 * 8) {
        float acc[16];
        const float* p = gu + (size_t)t * (2 * (size_t)F) + 2 * f0;
        for (int q = 0; q < 4; q++) {
            const float4 x = add_slices4(make_float4(0.f, 0.f, 0.f, 0.f), p + 4 * q, (size_t)T_pad * (2 * (size_t)F), n_split);
            acc[4 * q] = x.x;
            acc[4 * q + 1] = x.y;
            acc[4 * q + 2] = x.z;
            acc[4 * q + 3] = x.w;
        }
        float v[8];
        for (int i = 0; i < 8; i++) {
            const float g = acc[2 * i], u = acc[2 * i + 1];
            v[i] = g / (1.f + __expf(-g)) * u;
        }
        store_act8<BF16>(A, plane, t, f0, F, v);
    }
}

// externally produced K/V [n_layers, n_tok, Hkv, D] -> page slots of positions L .. L+n_tok-1
template <bool BF16>
__global__ void kv_ingest_kernel(const void* __restrict__ k_src, const void* __restrict__ v_src, int n_tok, int Hkv, int D,
                                 const int32_t* __restrict__ len_dev, int req_id, const int32_t* __restrict__ pages,
                                 void* __restrict__ k_pool, void* __restrict__ v_pool, int64_t n_pages) {
    const int tk = blockIdx.x, layer = blockIdx.y;
    const int pos = len_dev[req_id] + tk;
    const int page = pages[pos >> 4];
    const int slot = pos & 15;
    const size_t head_elems = (size_t)16 * D;
    for (int e = threadIdx.x; e < Hkv * D; e += blockDim.x) {
        const int g = e / D, dd = e - g * D;
        const size_t src = (((size_t)layer * n_tok + tk) * Hkv + g) * D + dd;
        const size_t base = (((size_t)layer * n_pages + page) * Hkv + g) * head_elems;
        if (BF16) {
            static_cast<bf16_t*>(k_pool)[base + kpage_offset(slot, dd)] = static_cast<const bf16_t*>(k_src)[src];
            static_cast<bf16_t*>(v_pool)[base + vpage_offset(slot, dd)] = static_cast<const bf16_t*>(v_src)[src];
        } else {
            static_cast<float*>(k_pool)[base + (size_t)slot * D + dd] = static_cast<const float*>(k_src)[src];
            static_cast<float*>(v_pool)[base + (size_t)slot * D + dd] = static_cast<const float*>(v_src)[src];
        }
    }
}

// the reverse: positions first .. first+n_tok-1 of a request -> [n_layers, n_tok, Hkv, D]
template <bool BF16>
__global__ void kv_export_kernel(void* __restrict__ k_dst, void* __restrict__ v_dst, int first, int n_tok, int Hkv, int D,
                                 const int32_t* __restrict__ pages, const void* __restrict__ k_pool,
                                 const void* __restrict__ v_pool, int64_t n_pages) {
    const int tk = blockIdx.x, layer = blockIdx.y;
    const int pos = first + tk;
    const int page = pages[pos >> 4];
    const int slot = pos & 15;
    const size_t head_elems = (size_t)16 * D;
    for (int e = threadIdx.x; e < Hkv * D; e += blockDim.x) {
        const int g = e / D, dd = e - g * D;
        const size_t dst = (((size_t)layer * n_tok + tk) * Hkv + g) * D + dd;
        const size_t base = (((size_t)layer * n_pages + page) * Hkv + g) * head_elems;
        if (BF16) {
            static_cast<bf16_t*>(k_dst)[dst] = static_cast<const bf16_t*>(k_pool)[base + kpage_offset(slot, dd)];
            static_cast<bf16_t*>(v_dst)[dst] = static_cast<const bf16_t*>(v_pool)[base + vpage_offset(slot, dd)];
        } else {
            static_cast<float*>(k_dst)[dst] = static_cast<const float*>(k_pool)[base + (size_t)slot * D + dd];
            static_cast<float*>(v_dst)[dst] = static_cast<const float*>(v_pool)[base + (size_t)slot * D + dd];
        }
    }
}

// row t of an activation buffer -> row 0 of another one
template <bool BF16>
__global__ __launch_bounds__(256) void copy_act_row_kernel(const void* __restrict__ X, size_t plane, int t, void* __restrict__ X1,
                                                           size_t plane1, int d) {
    for (int c = (blockIdx.x * 256 + threadIdx.x) * 8; c < d; c += gridDim.x * 256 * 8) {
        if (BF16) {
            const bf16_t* src = static_cast<const bf16_t*>(X) + frag_offset(t, c, d);
            bf16_t* dst = static_cast<bf16_t*>(X1) + frag_offset(0, c, d);
            *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
            *reinterpret_cast<uint4*>(dst + plane1) = *reinterpret_cast<const uint4*>(src + plane);
        } else {
            const float* src = static_cast<const float*>(X) + (size_t)t * d + c;
            float* dst = static_cast<float*>(X1) + c;
            *reinterpret_cast<float4*>(dst) = *reinterpret_cast<const float4*>(src);
            *reinterpret_cast<float4*>(dst + 4) = *reinterpret_cast<const float4*>(src + 4);
        }
    }
}

// len[req_ids[i]] += add[i]            (accept == nullptr)
// len[req_ids[i]] += accept[i] + 1     (otherwise)
__global__ void len_add_kernel(int32_t* __restrict__ len_dev, const int32_t* __restrict__ req_ids,
                               const int32_t* __restrict__ add, const int32_t* __restrict__ accept, int B) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B) return;
    len_dev[req_ids[i]] += accept ? accept[i] + 1 : add[i];
}

__global__ void fill_i32_kernel(int32_t* p, int32_t v, size_t n) {
    for (size_t e = blockIdx.x * (size_t)blockDim.x + threadIdx.x; e < n; e += (size_t)gridDim.x * blockDim.x) p[e] = v;
}

// ----- weight repacking --------------------------------------------------------------------
// rows [0, rows) of src[rows, K] go to destination rows dst_row0 + r * dst_row_stride of a packed
// (bf16, operand order) or row-major (f32) matrix with K columns.
template <bool BF16>
__global__ void pack_rows_kernel(const void* __restrict__ src, void* __restrict__ dst, int rows, int K, int dst_row0,
                                 int dst_row_stride, int dst_row_tiles) {
    const size_t n8 = (size_t)rows * (K / 8);
    for (size_t e = blockIdx.x * (size_t)blockDim.x + threadIdx.x; e < n8; e += (size_t)gridDim.x * blockDim.x) {
        const int r = (int)(e / (K / 8));
        const int c = (int)(e - (size_t)r * (K / 8)) * 8;
        const int dr = dst_row0 + r * dst_row_stride;
        if (BF16) {
            uint4 v = *reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(src) + (size_t)r * K + c);
            *reinterpret_cast<uint4*>(static_cast<bf16_t*>(dst) + wfrag_offset(dr, c, dst_row_tiles)) = v;
        } else {
            const float* s = static_cast<const float*>(src) + (size_t)r * K + c;
            float* d = static_cast<float*>(dst) + (size_t)dr * K + c;
            for (int i = 0; i < 8; i++) d[i] = s[i];
        }
    }
}

// rows of 8-bit weights (FP8 E4M3 bytes) -> paired-tile order
__global__ void pack_rows_w8_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst, int rows, int K, int dst_row0,
                                    int dst_row_stride, int dst_row_tiles) {
    const size_t n8 = (size_t)rows * (K / 8);
    for (size_t e = blockIdx.x * (size_t)blockDim.x + threadIdx.x; e < n8; e += (size_t)gridDim.x * blockDim.x) {
        const int r = (int)(e / (K / 8));
        const int c = (int)(e - (size_t)r * (K / 8)) * 8;
        const int dr = dst_row0 + r * dst_row_stride;
        const uint2 v = *reinterpret_cast<const uint2*>(src + (size_t)r * K + c);
        *reinterpret_cast<uint2*>(dst + w8_offset(dr, c, dst_row_tiles)) = v;
    }
}

// rows of packed FP4 codes [rows, K/2] -> paired-tile order; a thread moves 8 codes (4 bytes)
__global__ void pack_rows_w4_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst, int rows, int K, int dst_row0,
                                    int dst_row_stride, int dst_row_tiles) {
    const size_t n8 = (size_t)rows * (K / 8);
    for (size_t e = blockIdx.x * (size_t)blockDim.x + threadIdx.x; e < n8; e += (size_t)gridDim.x * blockDim.x) {
        const int r = (int)(e / (K / 8));
        const int c = (int)(e - (size_t)r * (K / 8)) * 8;
        const int dr = dst_row0 + r * dst_row_stride;
        const uint32_t v = *reinterpret_cast<const uint32_t*>(src + (size_t)r * (K / 2) + c / 2);
        *reinterpret_cast<uint32_t*>(dst + w4_offset(dr, c, dst_row_tiles)) = v;
    }
}

// their scale bytes [rows, K/32] -> interleaved order
__global__ void pack_scales_w4_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst, int rows, int KB, int dst_row0,
                                      int dst_row_stride, int dst_row_tiles) {
    const size_t n = (size_t)rows * KB;
    for (size_t e = blockIdx.x * (size_t)blockDim.x + threadIdx.x; e < n; e += (size_t)gridDim.x * blockDim.x) {
        const int r = (int)(e / KB);
        const int kb = (int)(e - (size_t)r * KB);
        dst[w4_scale_offset(dst_row0 + r * dst_row_stride, kb, dst_row_tiles)] = src[e];
    }
}

__global__ void scatter_scales_kernel(const float* __restrict__ src, float* __restrict__ dst, int rows, int dst_row0,
                                      int dst_row_stride) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < rows) dst[dst_row0 + i * dst_row_stride] = src[i];
}

template <bool BF16>
__global__ void copy_gain_kernel(const void* __restrict__ src, float* __restrict__ dst, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    dst[i] = BF16 ? bf16_to_f32(static_cast<const bf16_t*>(src)[i]) : static_cast<const float*>(src)[i];
}

}  // namespace

int sled_launch_pack_rows(int dtype, const void* src, void* dst, int rows, int K, int dst_row0, int dst_row_stride,
                          int dst_rows_total, hipStream_t st) {
    const int dst_row_tiles = dst_rows_total / 32;
    const size_t n8 = (size_t)rows * (K / 8);
    int grid = (int)((n8 + 255) / 256);
    if (grid > 65535) grid = 65535;
    if (grid < 1) grid = 1;
    if (dtype == SLED_BF16)
        hipLaunchKernelGGL(pack_rows_kernel<true>, dim3(grid), dim3(256), 0, st, src, dst, rows, K, dst_row0, dst_row_stride, dst_row_tiles);
    else
        hipLaunchKernelGGL(pack_rows_kernel<false>, dim3(grid), dim3(256), 0, st, src, dst, rows, K, dst_row0, dst_row_stride, dst_row_tiles);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

int sled_launch_pack_rows_w8(const void* src, void* dst, int rows, int K, int dst_row0, int dst_row_stride, int dst_rows_total,
                             hipStream_t st) {
    if (K % 16 || dst_rows_total % 64) SLED_FAIL(SLED_EINVAL, "8-bit weights: K %d or rows %d not tileable", K, dst_rows_total);
    const size_t n8 = (size_t)rows * (K / 8);
    int grid = (int)std::min<size_t>((n8 + 255) / 256, 65535);
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(pack_rows_w8_kernel, dim3(grid), dim3(256), 0, st, static_cast<const uint8_t*>(src), static_cast<uint8_t*>(dst),
                       rows, K, dst_row0, dst_row_stride, dst_rows_total / 32);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

int sled_launch_pack_rows_w4(const void* src, void* dst, int rows, int K, int dst_row0, int dst_row_stride, int dst_rows_total,
                             hipStream_t st) {
    if (K % 32 || dst_rows_total % 64) SLED_FAIL(SLED_EINVAL, "4-bit weights: K %d or rows %d not tileable", K, dst_rows_total);
    const size_t n8 = (size_t)rows * (K / 8);
    int grid = (int)std::min<size_t>((n8 + 255) / 256, 65535);
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(pack_rows_w4_kernel, dim3(grid), dim3(256), 0, st, static_cast<const uint8_t*>(src), static_cast<uint8_t*>(dst),
                       rows, K, dst_row0, dst_row_stride, dst_rows_total / 32);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

int sled_launch_pack_scales_w4(const void* src, void* dst, int rows, int K, int dst_row0, int dst_row_stride, int dst_rows_total,
                               hipStream_t st) {
    if (K % 32 || dst_rows_total % 64) SLED_FAIL(SLED_EINVAL, "4-bit weights: K %d or rows %d not tileable", K, dst_rows_total);
    const size_t n = (size_t)rows * (K / 32);
    int grid = (int)std::min<size_t>((n + 255) / 256, 65535);
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(pack_scales_w4_kernel, dim3(grid), dim3(256), 0, st, static_cast<const uint8_t*>(src),
                       static_cast<uint8_t*>(dst), rows, K / 32, dst_row0, dst_row_stride, dst_rows_total / 32);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

int sled_launch_scatter_scales(const float* src, float* dst, int rows, int dst_row0, int dst_row_stride, hipStream_t st) {
    hipLaunchKernelGGL(scatter_scales_kernel, dim3((rows + 255) / 256), dim3(256), 0, st, src, dst, rows, dst_row0, dst_row_stride);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

int sled_launch_copy_gain(int dtype, const void* src, float* dst, int n, hipStream_t st) {
    if (dtype == SLED_BF16)
        hipLaunchKernelGGL(copy_gain_kernel<true>, dim3((n + 255) / 256), dim3(256), 0, st, src, dst, n);
    else
        hipLaunchKernelGGL(copy_gain_kernel<false>, dim3((n + 255) / 256), dim3(256), 0, st, src, dst, n);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

int sled_launch_embed_norm(const sled_model* m, const int32_t* tokens, int T, float* h, void* X, size_t plane,
                           const float* gain, hipStream_t st) {
    if (m->s.dtype == SLED_BF16)
        hipLaunchKernelGGL(embed_norm_kernel<true>, dim3(T), dim3(256), 0, st, tokens, m->embed, m->s.vocab, m->s.d_model,
                           m->s.rms_eps, gain, h, X, plane);
    else
        hipLaunchKernelGGL(embed_norm_kernel<false>, dim3(T), dim3(256), 0, st, tokens, m->embed, m->s.vocab, m->s.d_model,
                           m->s.rms_eps, gain, h, X, plane);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

int sled_launch_residual_norm(const sled_model* m, const float* partial, int n_split, int T, int T_pad, float* h, void* X,
                              size_t plane, const float* gain, hipStream_t st) {
    // four columns per thread per trip: short rows get small workgroups
    const int bs = m->s.d_model >= 4096 ? 1024 : m->s.d_model >= 2048 ? 512 : m->s.d_model >= 1024 ? 256 : 128;
    if (m->s.dtype == SLED_BF16)
        hipLaunchKernelGGL(residual_norm_kernel<true>, dim3(T), dim3(bs), 0, st, partial, n_split, T_pad, m->s.d_model,
                           m->s.rms_eps, gain, h, X, plane);
    else
        hipLaunchKernelGGL(residual_norm_kernel<false>, dim3(T), dim3(bs), 0, st, partial, n_split, T_pad, m->s.d_model,
                           m->s.rms_eps, gain, h, X, plane);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

int sled_launch_copy_act_row(const sled_model* m, const void* X, size_t plane, int t, void* X1, size_t plane1, int d,
                             hipStream_t st) {
    if (d % 8) SLED_FAIL(SLED_EINVAL, "copy_act_row: d_model %d is not a multiple of 8", d);
    const int grid = (d / 8 + 255) / 256;
    if (m->s.dtype == SLED_BF16)
        hipLaunchKernelGGL(copy_act_row_kernel<true>, dim3(grid), dim3(256), 0, st, X, plane, t, X1, plane1, d);
    else
        hipLaunchKernelGGL(copy_act_row_kernel<false>, dim3(grid), dim3(256), 0, st, X, plane, t, X1, plane1, d);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

int sled_launch_rope_table(const sled_model* m, const sled_kvpool* p, const sled_step_meta& meta, float* cs, int32_t* kvslot,
                           hipStream_t st) {
    hipLaunchKernelGGL(rope_table_kernel, dim3(meta.T), dim3(64), 0, st, meta, p->len_dev, m->s.head_dim / 2,
                       (double)m->s.rope_theta, reinterpret_cast<float2*>(cs), kvslot);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

int sled_launch_attn_plan(const sled_model* m, const sled_kvpool* p, const sled_step_meta& meta, int32_t* plan, hipStream_t st) {
    hipLaunchKernelGGL(attn_plan_kernel, dim3((meta.n_work + 63) / 64), dim3(64), 0, st, meta, p->len_dev, m->s.n_kv_heads, plan);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

int sled_launch_qkv_rope_store(const sled_model* m, const sled_kvpool* p, int T, int layer, const float* partial, int n_split,
                               int T_pad, const float* cs, const int32_t* kvslot, void* Q, size_t q_plane, hipStream_t st) {
    const dim3 grid(T, m->s.n_q_heads + 2 * m->s.n_kv_heads);
    if (m->s.dtype == SLED_BF16)
        hipLaunchKernelGGL(qkv_rope_store_kernel<true>, grid, dim3(64), 0, st, partial, n_split, T_pad, m->s.n_q_heads,
                           m->s.n_kv_heads, m->s.head_dim, reinterpret_cast<const float2*>(cs), kvslot, Q, q_plane, p->k_pool,
                           p->v_pool, p->n_pages, layer);
    else
        hipLaunchKernelGGL(qkv_rope_store_kernel<false>, grid, dim3(64), 0, st, partial, n_split, T_pad, m->s.n_q_heads,
                           m->s.n_kv_heads, m->s.head_dim, reinterpret_cast<const float2*>(cs), kvslot, Q, q_plane, p->k_pool,
                           p->v_pool, p->n_pages, layer);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

int sled_launch_swiglu_reduce(const sled_model* m, const float* gu, int n_split, int T, int T_pad, void* A, size_t plane,
                              hipStream_t st) {
    const int F = m->s.d_ffn;
    int gy = (F / 8 + 255) / 256;
    if (gy > 8) gy = 8;
    if (gy < 1) gy = 1;
    dim3 grid(T, gy);
    if (m->s.dtype == SLED_BF16)
        hipLaunchKernelGGL(swiglu_reduce_kernel<true>, grid, dim3(256), 0, st, gu, n_split, T_pad, F, A, plane);
    else
        hipLaunchKernelGGL(swiglu_reduce_kernel<false>, grid, dim3(256), 0, st, gu, n_split, T_pad, F, A, plane);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

int sled_launch_kv_ingest(const sled_model* m, const sled_kvpool* p, const void* k_src, const void* v_src, int n_tokens,
                          int req_id, const int32_t* pages_dev, hipStream_t st) {
    dim3 grid(n_tokens, m->s.n_layers);
    if (m->s.dtype == SLED_BF16)
        hipLaunchKernelGGL(kv_ingest_kernel<true>, grid, dim3(256), 0, st, k_src, v_src, n_tokens, m->s.n_kv_heads,
                           m->s.head_dim, p->len_dev, req_id, pages_dev, p->k_pool, p->v_pool, p->n_pages);
    else
        hipLaunchKernelGGL(kv_ingest_kernel<false>, grid, dim3(256), 0, st, k_src, v_src, n_tokens, m->s.n_kv_heads,
                           m->s.head_dim, p->len_dev, req_id, pages_dev, p->k_pool, p->v_pool, p->n_pages);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

int sled_launch_kv_export(const sled_model* m, const sled_kvpool* p, void* k_dst, void* v_dst, int first, int n_tokens,
                          const int32_t* pages_dev, hipStream_t st) {
    dim3 grid(n_tokens, m->s.n_layers);
    if (m->s.dtype == SLED_BF16)
        hipLaunchKernelGGL(kv_export_kernel<true>, grid, dim3(256), 0, st, k_dst, v_dst, first, n_tokens, m->s.n_kv_heads,
                           m->s.head_dim, pages_dev, p->k_pool, p->v_pool, p->n_pages);
    else
        hipLaunchKernelGGL(kv_export_kernel<false>, grid, dim3(256), 0, st, k_dst, v_dst, first, n_tokens, m->s.n_kv_heads,
                           m->s.head_dim, pages_dev, p->k_pool, p->v_pool, p->n_pages);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

int sled_launch_len_add(int32_t* len_dev, const int32_t* req_ids_dev, const int32_t* add_dev, const int32_t* accept_dev,
                        int B, hipStream_t st) {
    hipLaunchKernelGGL(len_add_kernel, dim3((B + 63) / 64), dim3(64), 0, st, len_dev, req_ids_dev, add_dev, accept_dev, B);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}

int sled_launch_fill_i32(int32_t* p, int32_t v, size_t n, hipStream_t st) {
    int grid = (int)((n + 255) / 256);
    if (grid > 4096) grid = 4096;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(fill_i32_kernel, dim3(grid), dim3(256), 0, st, p, v, n);
    SLED_LAUNCH_CHECK();
    return SLED_OK;
}
