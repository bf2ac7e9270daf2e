// Internal declarations shared by the translation units of libsled (HIP, gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <vector>
#include <string>

#include "../../include/sled.h"

// ------------------------------------------------------------------------------------------
// error plumbing
// ------------------------------------------------------------------------------------------
void sled_set_error(const char* fmt, ...);

#define SLED_FAIL(code, ...)            \
    do {                                \
        sled_set_error(__VA_ARGS__);    \
        return (code);                  \
    } while (0)

#define SLED_HIP(expr)                                                                        \
    do {                                                                                      \
        hipError_t _e = (expr);                                                               \
        if (_e != hipSuccess)                                                                 \
            SLED_FAIL(SLED_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e), __FILE__, __LINE__); \
    } while (0)

#define SLED_LAUNCH_CHECK()                                                                   \
    do {                                                                                      \
        hipError_t _e = hipGetLastError();                                                    \
        if (_e != hipSuccess)                                                                 \
            SLED_FAIL(SLED_EHIP, "kernel launch failed: %s (%s:%d)", hipGetErrorString(_e), __FILE__, __LINE__); \
    } while (0)

// ------------------------------------------------------------------------------------------
// bf16 helpers (storage type is a raw 16-bit pattern; arithmetic is always fp32)
// ------------------------------------------------------------------------------------------
typedef uint16_t bf16_t;

__host__ __device__ inline float bf16_to_f32(bf16_t v) {
    union { uint32_t u; float f; } c;
    c.u = ((uint32_t)v) << 16;
    return c.f;
}

// round to nearest, ties to even; inputs are finite by contract
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
    union { uint32_t u; float f; } c;
    c.f = f;
    uint32_t u = c.u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// Rotation of one rotary pair (x1 = element i, x2 = element i + D/2) by the angle whose cosine and sine are c, s.
// Written with explicit roundings (one product, one fused multiply-add per output) so that every kernel that
// rotates gets the same bits whatever the compiler would otherwise contract.
__device__ inline void rope_pair(float x1, float x2, float c, float s, float& y1, float& y2) {
    y1 = __fmaf_rn(x1, c, -__fmul_rn(x2, s));
    y2 = __fmaf_rn(x2, c, __fmul_rn(x1, s));
}

// where element (token slot, dim dd) of a 16-token page of one kv head sits inside the page's 2048-element block
// of the bf16 pool: K in the operand order of S = K Q^T, V in the operand order of O = V^T P^T
__host__ __device__ inline int kpage_offset(int slot, int dd) { return (dd >> 5) * 512 + ((((dd & 31) >> 3) << 4) + slot) * 8 + (dd & 7); }
__host__ __device__ inline int vpage_offset(int slot, int dd) {
    const int dt = dd >> 4;
    return ((dt >> 1) * 64 + (slot >> 2) * 16 + (dd & 15)) * 8 + (dt & 1) * 4 + (slot & 3);
}

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short short4_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float float4_t;

// ------------------------------------------------------------------------------------------
// Packed operand layout for the bf16 projection kernels ("fragment order").
//
// A matrix M[R, K] (R = rows: output features of a weight, or tokens of an activation; K the
// contraction axis) is stored as tiles of 32 rows x 16 k.  A tile occupies 512 consecutive
// elements; inside it, lane l of a wavefront owns the 8 consecutive elements
//     M[rt*32 + l%32][ks*16 + (l/32)*8 + j],  j = 0..7
// which is exactly the operand register content of v_mfma_f32_32x32x16_bf16.  A wavefront
// therefore loads one operand tile with a single fully coalesced 1 KiB access.
// Activations order their tiles row-tile-major: tile (rt, ks) at (rt * K/16 + ks) * 512.
// ------------------------------------------------------------------------------------------
__host__ __device__ inline size_t frag_offset(int r, int k, int K) {
    int rt = r >> 5, rl = r & 31, ks = k >> 4, kk = k & 15;
    return ((size_t)rt * (K >> 4) + ks) * 512 + (size_t)(((kk >> 3) << 5) + rl) * 8 + (kk & 7);
}

// Weights use the same tiles, ordered k-step-major: tile (rt, ks) of a matrix with NT row tiles sits
// at (ks * NT + rt) * 512.  All wavefronts of a projection advance through k together, so at any
// moment the chip reads one contiguous window of NT KiB per k-step instead of thousands of streams
// a whole matrix row apart -- DRAM pages stay open.
__host__ __device__ inline size_t wfrag_offset(int r, int k, int NT) {
    int rt = r >> 5, rl = r & 31, ks = k >> 4, kk = k & 15;
    return ((size_t)ks * NT + rt) * 512 + (size_t)(((kk >> 3) << 5) + rl) * 8 + (kk & 7);
}

// 8-bit weights: byte offset of element (row r, column k) of a matrix with NT row tiles (NT even).  Two
// neighbouring row tiles share one 1 KiB block per k-step, so that a wavefront still fetches its two column tiles
// with one 16-byte-per-lane load: lane l = (k%16 / 8) * 32 + r%32 holds 8 k-values of tile 2p, then 8 of tile 2p+1.
__host__ __device__ inline size_t w8_offset(int r, int k, int NT) {
    const int pair = r >> 6, a = (r >> 5) & 1, rl = r & 31, ks = k >> 4, kk = k & 15;
    return ((size_t)ks * (NT >> 1) + pair) * 1024 + (size_t)(((kk >> 3) << 5) + rl) * 16 + a * 8 + (kk & 7);
}

// 4-bit weights (FP4 E2M1 codes, two per byte, with one power-of-two scale per row and block of 32 k -- the
// MXFP4 arrangement): byte offset of the byte that holds element (row r, column k); even k sit in the low nibble.
// As for 8 bits two neighbouring row tiles share a block per k-step, now 512 bytes: lane l = (k%16 / 8) * 32 + r%32
// holds 8 k-values of tile 2p in 4 bytes, then 8 of tile 2p+1.
__host__ __device__ inline size_t w4_offset(int r, int k, int NT) {
    const int pair = r >> 6, a = (r >> 5) & 1, rl = r & 31, ks = k >> 4, kk = k & 15;
    return ((size_t)ks * (NT >> 1) + pair) * 512 + (size_t)(((kk >> 3) << 5) + rl) * 8 + a * 4 + ((kk & 7) >> 1);
}
// ... and of the scale byte (E8M0: 2^(e - 127)) of row r and k-block kb = k / 32: the two tiles of a pair
// interleaved, so that a lane fetches both of its rows' scales with one 2-byte load
__host__ __device__ inline size_t w4_scale_offset(int r, int kb, int NT) {
    return ((size_t)kb * (NT >> 1) + (r >> 6)) * 64 + (size_t)(r & 31) * 2 + ((r >> 5) & 1);
}

// ------------------------------------------------------------------------------------------
// handles
// ------------------------------------------------------------------------------------------
struct sled_layer_weights {
    void* w_qkv;    // [ (Hq+2Hkv)*D, d ]  rows: q heads, then k heads, then v heads
    void* w_o;      // [ d, Hq*D ]
    void* w_gu;     // [ 2F, d ] row 2f = gate f, row 2f+1 = up f
    void* w_down;   // [ d, F ]
    float* g_attn;  // [d]
    float* g_mlp;   // [d]
    // 8-bit weights: one float scale per output row of each matrix (same row order as the matrix);
    // 4-bit weights: one scale byte per row and block of 32 k (w4_scale_offset)
    void* s_qkv = nullptr;
    void* s_o = nullptr;
    void* s_gu = nullptr;
    void* s_down = nullptr;
};

struct sled_model {
    sled_shape s;
    int n_qkv;                 // (Hq + 2 Hkv) * D
    size_t elem;               // bytes per stored element
    void* embed;               // [V, d] model dtype, row-major
    void* lm_head;             // [V, d] packed (bf16) or row-major (f32)
    float* g_final;
    std::vector<sled_layer_weights> layers;
    std::vector<void*> allocs;
    // bits per projection weight (sled_model_set_weight_bits): 16, 8 (FP8 E4M3, one scale per output row) or
    // 4 (FP4 E2M1, one power-of-two scale per row and 32 k)
    int wbits = 16;
    void* s_lm = nullptr;      // scales of the LM head
    // results of a request bit-identical whatever batch it is verified in (sled_model_set_batch_invariant)
    bool batch_invariant = false;
    // kernel timing (sled_profile_enable): one (class, start event, end event) per launch
    struct prof_span {
        int cls;
        hipEvent_t e0, e1;
    };
    bool prof_on = false;
    std::vector<prof_span> prof_spans;     // recorded since the last read
    std::vector<hipEvent_t> prof_free;     // events ready for reuse
};

struct sled_request {
    bool open = false;
    bool fresh = false;        // opened and not used yet: its device-side length is reset by the first call that has a stream
    int len_ub = 0;            // host-side upper bound of the committed length
    int staged = -1;           // k+1 of the last verify (rows staged), -1 if none
    int64_t added = 0;         // everything ever added to len_ub (lets a late read-back of the exact length be applied)
    uint32_t gen = 0;          // incarnation of the slot: a read-back taken for an earlier one is dropped
    std::vector<int> pages;
};

struct sled_kvpool {
    const sled_model* m;
    int64_t n_pages;
    int max_requests;
    size_t page_head_elems;    // 16 * head_dim
    void* k_pool;              // [n_layers][n_pages][Hkv][16*D] in the layout of the dtype
    void* v_pool;
    int32_t* len_dev;          // [max_requests] committed context length of each request
    std::vector<sled_request> reqs;
    std::vector<int> free_pages;
    std::vector<int> last_batch;   // request ids of the last verify
    // ring of pinned-host + device staging buffers for per-call metadata (page lists, row maps)
    static const int RING = 8;
    struct stage_slot {
        int32_t* host;
        int32_t* dev;
        hipEvent_t ev;
        bool pending;          // ev has been recorded and not yet waited for
    };
    stage_slot slot[RING];
    size_t stage_cap;          // ints per slot
    int stage_next;
    // Exact committed lengths come back asynchronously after a commit: a copy of len_dev into pinned memory and an
    // event behind it.  A later call that finds the event complete tightens the host-side bounds (and gives pages
    // back) without ever waiting.
    static const int READBACKS = 8;
    struct readback {
        int32_t* host = nullptr;          // pinned, max_requests ints
        hipEvent_t ev = nullptr;
        bool pending = false;
        std::vector<int> req;             // requests the commit touched
        std::vector<int64_t> added_at;    // their `added` right after that commit
        std::vector<uint32_t> gen_at;
    };
    readback rb[READBACKS];
    int rb_next = 0;
};

// per-step metadata blob, device side (offsets in int32 units from the blob start)
struct sled_step_meta {
    const int32_t* req_id;     // [B]   per row block of the step (a request has one, a prompt slice several)
    const int32_t* k;          // [B]   rows of the block - 1
    const int32_t* pos0;       // [B]   position of the block's first row behind the request's committed length
    const int32_t* cu_rows;    // [B+1]
    const int32_t* cu_pages;   // [B+1]
    const int32_t* row_req;    // [T]   index into the batch (not the request id)
    const int32_t* row_j;      // [T]   index of the row inside its request
    const int32_t* pages;      // [sum pages]
    const int32_t* work;       // [n_work * 4]  attention work items: batch index, kv head, first page, n pages
    const int32_t* cu_work;    // [B*Hkv][2]    first and end work item of each (batch index, kv head)
    int B, T, n_work;
};

// ------------------------------------------------------------------------------------------
// kernel launchers (defined in the .hip files); all return SLED_OK or an error code
// ------------------------------------------------------------------------------------------
// rowops.hip.  `plane` arguments: distance in elements between the hi and lo planes of an activation
// buffer of a bf16 model (unused for fp32 models).
int sled_launch_pack_rows(int dtype, const void* src, void* dst, int rows, int K, int dst_row0, int dst_row_stride,
                          int dst_rows_total, hipStream_t st);
int sled_launch_copy_gain(int dtype, const void* src, float* dst, int n, hipStream_t st);
// 8-bit weights: rows of an FP8 E4M3 matrix [rows, K] into the paired-tile order of w8_offset, and
// their float scales into the row order of the fused matrix
int sled_launch_pack_rows_w8(const void* src, void* dst, int rows, int K, int dst_row0, int dst_row_stride, int dst_rows_total,
                             hipStream_t st);
int sled_launch_scatter_scales(const float* src, float* dst, int rows, int dst_row0, int dst_row_stride, hipStream_t st);
// 4-bit weights: rows of packed FP4 codes [rows, K/2] into the order of w4_offset, and their scale bytes
// [rows, K/32] into the order of w4_scale_offset
int sled_launch_pack_rows_w4(const void* src, void* dst, int rows, int K, int dst_row0, int dst_row_stride, int dst_rows_total,
                             hipStream_t st);
int sled_launch_pack_scales_w4(const void* src, void* dst, int rows, int K, int dst_row0, int dst_row_stride, int dst_rows_total,
                               hipStream_t st);
// row t of an activation buffer -> row 0 of a one-tile buffer (the single row the LM head is asked for)
int sled_launch_copy_act_row(const sled_model* m, const void* X, size_t plane, int t, void* X1, size_t plane1, int d,
                             hipStream_t st);
int sled_launch_embed_norm(const sled_model* m, const int32_t* tokens, int T, float* h, void* X, size_t plane,
                           const float* gain, hipStream_t st);
int sled_launch_residual_norm(const sled_model* m, const float* partial, int n_split, int T, int T_pad, float* h, void* X,
                              size_t plane, const float* gain, hipStream_t st);
// per packed row: the rotary table cs[T][head_dim/2] and kvslot[T] = 16 * page + slot of the row's position in the cache
int sled_launch_rope_table(const sled_model* m, const sled_kvpool* p, const sled_step_meta& meta, float* cs, int32_t* kvslot,
                           hipStream_t st);
// one record of 12 ints per attention work item (see attn_plan_kernel)
int sled_launch_attn_plan(const sled_model* m, const sled_kvpool* p, const sled_step_meta& meta, int32_t* plan, hipStream_t st);
int sled_launch_qkv_rope_store(const sled_model* m, const sled_kvpool* p, int T, int layer, const float* partial, int n_split,
                               int T_pad, const float* cs, const int32_t* kvslot, void* Q, size_t q_plane, hipStream_t st);
int sled_launch_swiglu_reduce(const sled_model* m, const float* gu, int n_split, int T, int T_pad, void* A, size_t plane,
                              hipStream_t st);
int sled_launch_kv_ingest(const sled_model* m, const sled_kvpool* p, const void* k_src, const void* v_src, int n_tokens,
                          int req_id, const int32_t* pages_dev, hipStream_t st);
int sled_launch_kv_export(const sled_model* m, const sled_kvpool* p, void* k_dst, void* v_dst, int first, int n_tokens,
                          const int32_t* pages_dev, hipStream_t st);
int sled_launch_len_add(int32_t* len_dev, const int32_t* req_ids_dev, const int32_t* add_dev, const int32_t* accept_dev,
                        int B, hipStream_t st);

// gemm.hip:  out = X[T, K] * W[N, K]^T
enum { SLED_EPI_PARTIAL = 0, SLED_EPI_SWIGLU = 1, SLED_EPI_STORE = 2 };
struct sled_gemm_plan {
    int split;   // K slices
    int cap;     // the most K slices a step may choose instead (sizes the partial-sum buffer)
};
sled_gemm_plan sled_gemm_make_plan(const sled_model* m, int N, int K, bool needs_full_k);
// the plan for a step of T_pad rows: never more K slices than `base` (which sizes the workspace), fewer where several
// blocks of rows already give every CU a workgroup
sled_gemm_plan sled_gemm_plan_rows(const sled_model* m, sled_gemm_plan base, int N, int K, int T_pad);
// `scale`: the scales of an 8-bit or 4-bit weight matrix (models with such weights), else nullptr
int sled_launch_gemm(const sled_model* m, const void* X, size_t x_plane, const void* W, const void* scale, int T, int T_pad,
                     int N, int K, int epilogue, sled_gemm_plan plan, float* out_f32, void* out_act, size_t act_plane,
                     int F_act, hipStream_t st);

// attention.hip
// qkv_partial != nullptr (bf16 models, every block a request of its own): the kernel itself adds up the K slices of the
// QKV projection, rotates q and k and writes the new K/V rows into the cache; Q is then not read.
int sled_launch_attention(const sled_model* m, const sled_kvpool* p, const sled_step_meta& meta, int layer, const void* Q,
                          size_t q_plane, const float* qkv_partial, int n_split, int T_pad, const float* cs,
                          const int32_t* kvslot, const int32_t* plan, float* part_o, float* part_ml, int32_t* arrive,
                          void* X_out, size_t x_plane, int QT, hipStream_t st);
int sled_launch_fill_i32(int32_t* p, int32_t v, size_t n, hipStream_t st);

// accept.hip
size_t sled_accept_ws_bytes(int B, int T, int n_split);
int sled_accept_pick_split(int T, int vocab);
int sled_launch_row_confidence(int T, int vocab, float temperature, const float* logits, float* conf, int32_t* top, void* ws,
                               hipStream_t st);
int sled_launch_accept(int mode, int B, int T, const int* k_host, int vocab, float temperature, const float* logits,
                       const int32_t* tokens, const float* draft_q, const int32_t* q_ids, const float* q_probs,
                       const float* q_rest, int q_m, const float* u_acc, const float* u_smp, int32_t* accept_len, int32_t* out_token, void* ws,
                       hipStream_t st);
