// Host side of libsled: handles, argument checks, page accounting, the per-step metadata blob
// (ragged packing: row -> request map, page lists, attention work list) and the launch sequence
// of one verification step.  No device work is done here except enqueueing kernels and copies.
#include "sled_internal.h"

#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include <algorithm>
#include <new>

// ------------------------------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";

void sled_set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

extern "C" const char* sled_last_error(void) { return g_err; }

extern "C" const char* sled_strerror(int code) {
    switch (code) {
        case SLED_OK: return "ok";
        case SLED_EINVAL: return "invalid argument";
        case SLED_ENOMEM: return "out of pages, request slots or memory";
        case SLED_ESTATE: return "call out of order";
        case SLED_EHIP: return "HIP runtime error";
        default: return "unknown error";
    }
}

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// ------------------------------------------------------------------------------------------ model
static int model_alloc(sled_model* m, void** out, size_t bytes) {
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) SLED_FAIL(SLED_ENOMEM, "hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
    m->allocs.push_back(p);
    *out = p;
    return SLED_OK;
}

// replaces the allocation *p by one of `bytes` bytes (contents are not kept)
static int model_resize(sled_model* m, void** p, size_t bytes) {
    for (size_t i = 0; i < m->allocs.size(); i++)
        if (m->allocs[i] == *p) {
            (void)hipFree(*p);
            m->allocs.erase(m->allocs.begin() + i);
            break;
        }
    *p = nullptr;
    return model_alloc(m, p, bytes);
}

extern "C" int sled_model_create(const sled_shape* shape, sled_model** out) {
    if (!shape || !out) SLED_FAIL(SLED_EINVAL, "sled_model_create: null argument");
    const sled_shape& s = *shape;
    if (s.n_layers < 1 || s.d_model < 8 || s.n_q_heads < 1 || s.n_kv_heads < 1 || s.head_dim < 2 || s.d_ffn < 8 ||
        s.vocab < 2)
        SLED_FAIL(SLED_EINVAL, "sled_model_create: non-positive dimension");
    if (s.n_q_heads % s.n_kv_heads) SLED_FAIL(SLED_EINVAL, "n_q_heads must be a multiple of n_kv_heads");
    if (s.page_size != 16) SLED_FAIL(SLED_EINVAL, "page_size must be 16");
    if (s.k_max < 0 || s.k_max > 15) SLED_FAIL(SLED_EINVAL, "k_max must be in [0, 15]");
    if (!(s.rms_eps >= 0.f) || !(s.rope_theta > 0.f)) SLED_FAIL(SLED_EINVAL, "bad rms_eps or rope_theta");
    const int G = s.n_q_heads / s.n_kv_heads;
    if (s.dtype == SLED_BF16) {
        if (s.head_dim != 128) SLED_FAIL(SLED_EINVAL, "bf16 models need head_dim 128");
        if (s.d_model % 256 || s.d_ffn % 256 || (s.n_q_heads * s.head_dim) % 256)
            SLED_FAIL(SLED_EINVAL, "bf16 models need d_model, d_ffn and n_q_heads*head_dim multiples of 256");
        if (s.vocab % 32) SLED_FAIL(SLED_EINVAL, "bf16 models need vocab a multiple of 32");
        if (G * (s.k_max + 1) > 80) SLED_FAIL(SLED_EINVAL, "(n_q_heads/n_kv_heads)*(k_max+1) must be <= 80");
    } else if (s.dtype == SLED_F32) {
        if (s.head_dim != 64 && s.head_dim != 128) SLED_FAIL(SLED_EINVAL, "fp32 models need head_dim 64 or 128");
        if (s.d_model % 8 || s.d_ffn % 8) SLED_FAIL(SLED_EINVAL, "fp32 models need d_model and d_ffn multiples of 8");
    } else {
        SLED_FAIL(SLED_EINVAL, "unknown dtype %d", s.dtype);
    }
    sled_model* m = new (std::nothrow) sled_model();
    if (!m) SLED_FAIL(SLED_ENOMEM, "host allocation failed");
    m->s = s;
    m->elem = s.dtype == SLED_BF16 ? 2 : 4;
    m->n_qkv = (s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim;
    const size_t d = s.d_model, F = s.d_ffn, V = s.vocab, HD = (size_t)s.n_q_heads * s.head_dim;
    int rc = SLED_OK;
    auto A = [&](void** p, size_t bytes) {
        if (rc == SLED_OK) rc = model_alloc(m, p, bytes);
    };
    A(&m->embed, V * d * m->elem);
    A(&m->lm_head, V * d * m->elem);
    A(reinterpret_cast<void**>(&m->g_final), d * sizeof(float));
    m->layers.resize(s.n_layers);
    for (int l = 0; l < s.n_layers && rc == SLED_OK; l++) {
        sled_layer_weights& w = m->layers[l];
        A(&w.w_qkv, (size_t)m->n_qkv * d * m->elem);
        A(&w.w_o, d * HD * m->elem);
        A(&w.w_gu, 2 * F * d * m->elem);
        A(&w.w_down, d * F * m->elem);
        A(reinterpret_cast<void**>(&w.g_attn), d * sizeof(float));
        A(reinterpret_cast<void**>(&w.g_mlp), d * sizeof(float));
    }
    if (rc != SLED_OK) {
        sled_model_destroy(m);
        return rc;
    }
    *out = m;
    return SLED_OK;
}

extern "C" int sled_model_destroy(sled_model* m) {
    if (!m) return SLED_OK;
    (void)hipDeviceSynchronize();
    for (auto& sp : m->prof_spans) {
        (void)hipEventDestroy(sp.e0);
        (void)hipEventDestroy(sp.e1);
    }
    for (hipEvent_t e : m->prof_free) (void)hipEventDestroy(e);
    for (void* p : m->allocs) (void)hipFree(p);
    delete m;
    return SLED_OK;
}

extern "C" int sled_model_load(sled_model* m, int tensor_id, int layer, const void* src, void* stream) {
    if (!m || !src) SLED_FAIL(SLED_EINVAL, "sled_model_load: null argument");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const sled_shape& s = m->s;
    const int d = s.d_model, F = s.d_ffn, D = s.head_dim, HD = s.n_q_heads * D, KD = s.n_kv_heads * D;
    const bool per_layer = tensor_id >= SLED_T_WQ && tensor_id <= SLED_T_G_MLP;
    if (per_layer && (layer < 0 || layer >= s.n_layers)) SLED_FAIL(SLED_EINVAL, "sled_model_load: layer %d out of range", layer);
    if (tensor_id >= SLED_T_SCALE) {
        // scales of an 8-bit matrix: float32 [rows]; of a 4-bit matrix: one byte per row and 32 k, [rows, K/32];
        // both go into the row order of the fused matrix
        const int mat = tensor_id - SLED_T_SCALE;
        if (m->wbits == 16) SLED_FAIL(SLED_EINVAL, "sled_model_load: scales given to a model with 16-bit weights");
        const bool lay = mat >= SLED_T_WQ && mat <= SLED_T_WDOWN;
        if (lay && (layer < 0 || layer >= s.n_layers)) SLED_FAIL(SLED_EINVAL, "sled_model_load: layer %d out of range", layer);
        sled_layer_weights* ws = lay ? &m->layers[layer] : nullptr;
        auto put = [&](void* dst, int rows, int K, int row0, int stride, int rows_total) {
            if (m->wbits == 8) return sled_launch_scatter_scales(static_cast<const float*>(src), static_cast<float*>(dst), rows, row0, stride, st);
            return sled_launch_pack_scales_w4(src, dst, rows, K, row0, stride, rows_total, st);
        };
        switch (mat) {
            case SLED_T_WQ: return put(ws->s_qkv, HD, d, 0, 1, m->n_qkv);
            case SLED_T_WK: return put(ws->s_qkv, KD, d, HD, 1, m->n_qkv);
            case SLED_T_WV: return put(ws->s_qkv, KD, d, HD + KD, 1, m->n_qkv);
            case SLED_T_WO: return put(ws->s_o, d, HD, 0, 1, d);
            case SLED_T_WGATE: return put(ws->s_gu, F, d, 0, 2, 2 * F);
            case SLED_T_WUP: return put(ws->s_gu, F, d, 1, 2, 2 * F);
            case SLED_T_WDOWN: return put(ws->s_down, d, F, 0, 1, d);
            case SLED_T_LM_HEAD: return put(m->s_lm, s.vocab, d, 0, 1, s.vocab);
            default: SLED_FAIL(SLED_EINVAL, "sled_model_load: tensor %d has no scales", mat);
        }
    }
    sled_layer_weights* w = per_layer ? &m->layers[layer] : nullptr;
    if (m->wbits != 16) {
        // matrices arrive as FP8 E4M3 bytes [out, in], or as FP4 E2M1 codes, two per byte, [out, in / 2]
        auto put = [&](void* dst, int rows, int K, int row0, int stride, int rows_total) {
            if (m->wbits == 8) return sled_launch_pack_rows_w8(src, dst, rows, K, row0, stride, rows_total, st);
            return sled_launch_pack_rows_w4(src, dst, rows, K, row0, stride, rows_total, st);
        };
        switch (tensor_id) {
            case SLED_T_WQ: return put(w->w_qkv, HD, d, 0, 1, m->n_qkv);
            case SLED_T_WK: return put(w->w_qkv, KD, d, HD, 1, m->n_qkv);
            case SLED_T_WV: return put(w->w_qkv, KD, d, HD + KD, 1, m->n_qkv);
            case SLED_T_WO: return put(w->w_o, d, HD, 0, 1, d);
            case SLED_T_WGATE: return put(w->w_gu, F, d, 0, 2, 2 * F);
            case SLED_T_WUP: return put(w->w_gu, F, d, 1, 2, 2 * F);
            case SLED_T_WDOWN: return put(w->w_down, d, F, 0, 1, d);
            case SLED_T_LM_HEAD: return put(m->lm_head, s.vocab, d, 0, 1, s.vocab);
            default: break;  // embedding and gains as in a 16-bit model
        }
    }
    switch (tensor_id) {
        case SLED_T_EMBED:
            SLED_HIP(hipMemcpyAsync(m->embed, src, (size_t)s.vocab * d * m->elem, hipMemcpyDeviceToDevice, st));
            return SLED_OK;
        case SLED_T_WQ: return sled_launch_pack_rows(s.dtype, src, w->w_qkv, HD, d, 0, 1, m->n_qkv, st);
        case SLED_T_WK: return sled_launch_pack_rows(s.dtype, src, w->w_qkv, KD, d, HD, 1, m->n_qkv, st);
        case SLED_T_WV: return sled_launch_pack_rows(s.dtype, src, w->w_qkv, KD, d, HD + KD, 1, m->n_qkv, st);
        case SLED_T_WO: return sled_launch_pack_rows(s.dtype, src, w->w_o, d, HD, 0, 1, d, st);
        case SLED_T_WGATE: return sled_launch_pack_rows(s.dtype, src, w->w_gu, F, d, 0, 2, 2 * F, st);
        case SLED_T_WUP: return sled_launch_pack_rows(s.dtype, src, w->w_gu, F, d, 1, 2, 2 * F, st);
        case SLED_T_WDOWN: return sled_launch_pack_rows(s.dtype, src, w->w_down, d, F, 0, 1, d, st);
        case SLED_T_G_ATTN: return sled_launch_copy_gain(s.dtype, src, w->g_attn, d, st);
        case SLED_T_G_MLP: return sled_launch_copy_gain(s.dtype, src, w->g_mlp, d, st);
        case SLED_T_G_FINAL: return sled_launch_copy_gain(s.dtype, src, m->g_final, d, st);
        case SLED_T_LM_HEAD: return sled_launch_pack_rows(s.dtype, src, m->lm_head, s.vocab, d, 0, 1, s.vocab, st);
        default: SLED_FAIL(SLED_EINVAL, "sled_model_load: unknown tensor id %d", tensor_id);
    }
}

// ------------------------------------------------------------------------------------------ timing
static int prof_event(sled_model* m, hipEvent_t* out) {
    if (!m->prof_free.empty()) {
        *out = m->prof_free.back();
        m->prof_free.pop_back();
        return SLED_OK;
    }
    SLED_HIP(hipEventCreate(out));
    return SLED_OK;
}

// brackets one launch (or a short group of launches of the same class) with events
struct prof_scope {
    sled_model* m;
    hipStream_t st;
    sled_model::prof_span sp;
    bool live;
    prof_scope(sled_model* m_, int cls, hipStream_t st_) : m(m_), st(st_), live(false) {
        if (!m->prof_on) return;
        sp.cls = cls;
        if (prof_event(m, &sp.e0) != SLED_OK || prof_event(m, &sp.e1) != SLED_OK) return;
        live = hipEventRecord(sp.e0, st) == hipSuccess;
    }
    ~prof_scope() {
        if (!live) return;
        (void)hipEventRecord(sp.e1, st);
        m->prof_spans.push_back(sp);
    }
};

extern "C" int sled_model_set_weight_bits(sled_model* m, int bits) {
    if (!m) SLED_FAIL(SLED_EINVAL, "sled_model_set_weight_bits: null model");
    if (bits != 16 && bits != 8 && bits != 4) SLED_FAIL(SLED_EINVAL, "sled_model_set_weight_bits: %d bits unsupported (16, 8 or 4)", bits);
    const sled_shape& s = m->s;
    if (bits == 16 && s.dtype != SLED_BF16) return SLED_OK;  // an fp32 model has no other format
    if (s.dtype != SLED_BF16) SLED_FAIL(SLED_EINVAL, "sled_model_set_weight_bits: 8- and 4-bit weights need a bf16 model");
    if (bits != 16 && (m->n_qkv % 64 || s.d_model % 64 || (2 * s.d_ffn) % 64 || s.vocab % 64))
        SLED_FAIL(SLED_EINVAL, "sled_model_set_weight_bits: output widths must be multiples of 64");
    if (bits != m->wbits) {
        // the projection matrices take bits/8 bytes per weight: give back what the previous format held
        SLED_HIP(hipDeviceSynchronize());
        int rc = SLED_OK;
        auto R = [&](void** p, size_t rows, size_t K) {
            if (rc == SLED_OK) rc = model_resize(m, p, rows * K * bits / 8);
        };
        const size_t d = s.d_model, HD = (size_t)s.n_q_heads * s.head_dim, F = s.d_ffn;
        R(&m->lm_head, s.vocab, d);
        for (auto& w : m->layers) {
            R(&w.w_qkv, m->n_qkv, d);
            R(&w.w_o, d, HD);
            R(&w.w_gu, 2 * F, d);
            R(&w.w_down, d, F);
        }
        if (rc != SLED_OK) return rc;  // the model is unusable now: destroy it
        m->wbits = bits;
    }
    if (bits == 16) return SLED_OK;
    if (!m->s_lm) {
        // room for either kind of scales: a float per row, or a byte per row and 32 k
        int rc = SLED_OK;
        auto A = [&](void** p, size_t rows, size_t K) {
            if (rc == SLED_OK) rc = model_alloc(m, p, std::max(rows * sizeof(float), rows * (K / 32)));
        };
        const size_t d = s.d_model, HD = (size_t)s.n_q_heads * s.head_dim;
        A(&m->s_lm, s.vocab, d);
        for (auto& w : m->layers) {
            A(&w.s_qkv, m->n_qkv, d);
            A(&w.s_o, d, HD);
            A(&w.s_gu, 2 * (size_t)s.d_ffn, d);
            A(&w.s_down, d, s.d_ffn);
        }
        if (rc != SLED_OK) return rc;
    }
    m->wbits = bits;
    return SLED_OK;
}

extern "C" int sled_model_set_batch_invariant(sled_model* m, int on) {
    if (!m) SLED_FAIL(SLED_EINVAL, "sled_model_set_batch_invariant: null model");
    m->batch_invariant = on != 0;
    return SLED_OK;
}

extern "C" int sled_profile_enable(sled_model* m, int on) {
    if (!m) SLED_FAIL(SLED_EINVAL, "sled_profile_enable: null model");
    m->prof_on = on != 0;
    return SLED_OK;
}

extern "C" int sled_profile_read(sled_model* m, void* stream, float* ms, int* launches) {
    if (!m || !ms || !launches) SLED_FAIL(SLED_EINVAL, "sled_profile_read: null argument");
    SLED_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
    for (int c = 0; c < SLED_PROF_N; c++) {
        ms[c] = 0.f;
        launches[c] = 0;
    }
    for (auto& sp : m->prof_spans) {
        float t = 0.f;
        SLED_HIP(hipEventElapsedTime(&t, sp.e0, sp.e1));
        ms[sp.cls] += t;
        launches[sp.cls] += 1;
        m->prof_free.push_back(sp.e0);
        m->prof_free.push_back(sp.e1);
    }
    m->prof_spans.clear();
    return SLED_OK;
}

// ------------------------------------------------------------------------------------------ pool
typedef sled_kvpool::stage_slot sled_stage_slot;

static int slot_alloc(sled_stage_slot& s, size_t cap) {
    SLED_HIP(hipHostMalloc(reinterpret_cast<void**>(&s.host), cap * sizeof(int32_t), hipHostMallocDefault));
    SLED_HIP(hipMalloc(reinterpret_cast<void**>(&s.dev), cap * sizeof(int32_t)));
    return SLED_OK;
}

// next staging slot with room for n ints; waits until the work that last used it has finished
static int stage_acquire(sled_kvpool* p, size_t n, sled_stage_slot** out) {
    sled_kvpool* pv = p;
    if (n > pv->stage_cap) {
        // grow every slot (rare: only when a batch is larger than anything seen before)
        size_t cap = std::max(n, pv->stage_cap * 2);
        for (int i = 0; i < sled_kvpool::RING; i++) {
            sled_stage_slot& s = pv->slot[i];
            if (s.pending) SLED_HIP(hipEventSynchronize(s.ev));
            s.pending = false;
            (void)hipHostFree(s.host);
            (void)hipFree(s.dev);
            int rc = slot_alloc(s, cap);
            if (rc != SLED_OK) return rc;
        }
        pv->stage_cap = cap;
    }
    sled_stage_slot& s = pv->slot[pv->stage_next];
    pv->stage_next = (pv->stage_next + 1) % sled_kvpool::RING;
    if (s.pending) SLED_HIP(hipEventSynchronize(s.ev));
    s.pending = false;
    *out = &s;
    return SLED_OK;
}

static int stage_release(sled_stage_slot* s, hipStream_t st) {
    SLED_HIP(hipEventRecord(s->ev, st));
    s->pending = true;
    return SLED_OK;
}

extern "C" int sled_kvpool_create(const sled_model* m, int64_t n_pages, int max_requests, sled_kvpool** out) {
    if (!m || !out || n_pages < 1 || max_requests < 1) SLED_FAIL(SLED_EINVAL, "sled_kvpool_create: bad argument");
    // 16 * page + slot is kept in 32 bits
    if (n_pages > (int64_t)1 << 27) SLED_FAIL(SLED_EINVAL, "sled_kvpool_create: too many pages");
    sled_kvpool* p = new (std::nothrow) sled_kvpool();
    if (!p) SLED_FAIL(SLED_ENOMEM, "host allocation failed");
    p->m = m;
    p->n_pages = n_pages;
    p->max_requests = max_requests;
    p->page_head_elems = (size_t)16 * m->s.head_dim;
    p->k_pool = p->v_pool = nullptr;
    p->len_dev = nullptr;
    for (int i = 0; i < sled_kvpool::RING; i++) p->slot[i] = sled_stage_slot{nullptr, nullptr, nullptr, false};
    p->stage_cap = 0;
    p->stage_next = 0;
    const size_t bytes = (size_t)m->s.n_layers * n_pages * m->s.n_kv_heads * p->page_head_elems * m->elem;
    auto fail = [&](int code, const char* what, hipError_t e) {
        sled_set_error("sled_kvpool_create: %s failed: %s", what, hipGetErrorString(e));
        sled_kvpool_destroy(p);
        return code;
    };
    hipError_t e;
    if ((e = hipMalloc(&p->k_pool, bytes)) != hipSuccess) return fail(SLED_ENOMEM, "hipMalloc(K pool)", e);
    if ((e = hipMalloc(&p->v_pool, bytes)) != hipSuccess) return fail(SLED_ENOMEM, "hipMalloc(V pool)", e);
    if ((e = hipMalloc(reinterpret_cast<void**>(&p->len_dev), max_requests * sizeof(int32_t))) != hipSuccess)
        return fail(SLED_ENOMEM, "hipMalloc(lengths)", e);
    // pages never written hold zeros (read only under the mask, but keep them finite)
    if ((e = hipMemset(p->k_pool, 0, bytes)) != hipSuccess) return fail(SLED_EHIP, "hipMemset", e);
    if ((e = hipMemset(p->v_pool, 0, bytes)) != hipSuccess) return fail(SLED_EHIP, "hipMemset", e);
    if ((e = hipMemset(p->len_dev, 0, max_requests * sizeof(int32_t))) != hipSuccess) return fail(SLED_EHIP, "hipMemset", e);
    p->stage_cap = 1 << 16;
    for (int i = 0; i < sled_kvpool::RING; i++) {
        if (slot_alloc(p->slot[i], p->stage_cap) != SLED_OK) {
            sled_kvpool_destroy(p);
            return SLED_ENOMEM;
        }
        if ((e = hipEventCreateWithFlags(&p->slot[i].ev, hipEventDisableTiming)) != hipSuccess)
            return fail(SLED_EHIP, "hipEventCreate", e);
    }
    for (int i = 0; i < sled_kvpool::READBACKS; i++) {
        if ((e = hipHostMalloc(reinterpret_cast<void**>(&p->rb[i].host), max_requests * sizeof(int32_t), hipHostMallocDefault)) != hipSuccess)
            return fail(SLED_ENOMEM, "hipHostMalloc(length read-back)", e);
        if ((e = hipEventCreateWithFlags(&p->rb[i].ev, hipEventDisableTiming)) != hipSuccess)
            return fail(SLED_EHIP, "hipEventCreate", e);
    }
    if ((e = hipDeviceSynchronize()) != hipSuccess) return fail(SLED_EHIP, "hipDeviceSynchronize", e);
    p->reqs.resize(max_requests);
    p->free_pages.reserve(n_pages);
    for (int64_t i = n_pages - 1; i >= 0; i--) p->free_pages.push_back((int)i);
    *out = p;
    return SLED_OK;
}

extern "C" int sled_kvpool_destroy(sled_kvpool* p) {
    if (!p) return SLED_OK;
    (void)hipDeviceSynchronize();
    for (int i = 0; i < sled_kvpool::RING; i++) {
        if (p->slot[i].host) (void)hipHostFree(p->slot[i].host);
        if (p->slot[i].dev) (void)hipFree(p->slot[i].dev);
        if (p->slot[i].ev) (void)hipEventDestroy(p->slot[i].ev);
    }
    for (int i = 0; i < sled_kvpool::READBACKS; i++) {
        if (p->rb[i].host) (void)hipHostFree(p->rb[i].host);
        if (p->rb[i].ev) (void)hipEventDestroy(p->rb[i].ev);
    }
    if (p->k_pool) (void)hipFree(p->k_pool);
    if (p->v_pool) (void)hipFree(p->v_pool);
    if (p->len_dev) (void)hipFree(p->len_dev);
    delete p;
    return SLED_OK;
}

extern "C" int sled_kvpool_open(sled_kvpool* p, int* req_id) {
    if (!p || !req_id) SLED_FAIL(SLED_EINVAL, "sled_kvpool_open: null argument");
    for (int i = 0; i < p->max_requests; i++)
        if (!p->reqs[i].open) {
            // A closed slot's device-side length may be stale.  This call has no stream, so nothing is enqueued
            // here: the first append, verify or prefill that names the request resets the length on its own stream
            // before anything reads it (reset_fresh_lengths).
            const uint32_t gen = p->reqs[i].gen + 1;
            p->reqs[i] = sled_request();
            p->reqs[i].open = true;
            p->reqs[i].fresh = true;
            p->reqs[i].gen = gen;
            *req_id = i;
            return SLED_OK;
        }
    SLED_FAIL(SLED_ENOMEM, "sled_kvpool_open: all %d request slots are in use", p->max_requests);
}

extern "C" int sled_kvpool_close(sled_kvpool* p, int req_id) {
    if (!p || req_id < 0 || req_id >= p->max_requests || !p->reqs[req_id].open)
        SLED_FAIL(SLED_EINVAL, "sled_kvpool_close: request %d is not open", req_id);
    // No wait: work that still reads these pages was enqueued earlier on the pool's stream, and whoever is handed
    // the pages next writes them from a later call on that stream (calls on one pool share a stream or are ordered
    // by the caller).
    for (int pg : p->reqs[req_id].pages) p->free_pages.push_back(pg);
    const uint32_t gen = p->reqs[req_id].gen;
    p->reqs[req_id] = sled_request();
    p->reqs[req_id].gen = gen;
    p->last_batch.erase(std::remove(p->last_batch.begin(), p->last_batch.end(), req_id), p->last_batch.end());
    return SLED_OK;
}

// pages a request has to keep: its committed tokens (upper bound) and the rows a verify has staged behind them
static void trim_pages(sled_kvpool* p, sled_request& rq) {
    const int keep = ceil_div(rq.len_ub + std::max(rq.staged, 0), 16);
    while ((int)rq.pages.size() > keep) {
        p->free_pages.push_back(rq.pages.back());
        rq.pages.pop_back();
    }
}

// Applies every length read-back whose copy has completed (never waits): the exact length L of a request right after
// some commit, plus whatever has been added to its bound since, is a tighter bound than the one kept so far.
static void poll_readbacks(sled_kvpool* p) {
    for (int n = 0; n < sled_kvpool::READBACKS; n++) {
        sled_kvpool::readback& rb = p->rb[(p->rb_next + n) % sled_kvpool::READBACKS];   // oldest first
        if (!rb.pending) continue;
        if (hipEventQuery(rb.ev) != hipSuccess) {
            (void)hipGetLastError();   // hipErrorNotReady is not an error
            continue;
        }
        rb.pending = false;
        for (size_t i = 0; i < rb.req.size(); i++) {
            sled_request& rq = p->reqs[rb.req[i]];
            if (!rq.open || rq.gen != rb.gen_at[i]) continue;
            const int64_t ub = (int64_t)rb.host[rb.req[i]] + (rq.added - rb.added_at[i]);
            if (ub < rq.len_ub) {
                rq.len_ub = (int)ub;
                trim_pages(p, rq);
            }
        }
    }
}

// the device-side length of a request that has just been opened is reset here, on the first stream that names it
static int reset_fresh_lengths(sled_kvpool* p, int B, const int* req_ids, hipStream_t st) {
    for (int i = 0; i < B; i++) {
        sled_request& rq = p->reqs[req_ids[i]];
        if (!rq.fresh) continue;
        int rc = sled_launch_fill_i32(p->len_dev + req_ids[i], 0, 1, st);
        if (rc != SLED_OK) return rc;
        rq.fresh = false;
    }
    return SLED_OK;
}

// after a commit: copy the lengths back behind it, to be looked at by a later call
static int enqueue_readback(sled_kvpool* p, int B, const int* req_ids, hipStream_t st) {
    sled_kvpool::readback& rb = p->rb[p->rb_next];
    if (rb.pending) return SLED_OK;   // the ring is full of copies nobody has looked at yet: skip this one
    SLED_HIP(hipMemcpyAsync(rb.host, p->len_dev, p->max_requests * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    SLED_HIP(hipEventRecord(rb.ev, st));
    rb.req.assign(req_ids, req_ids + B);
    rb.added_at.resize(B);
    rb.gen_at.resize(B);
    for (int i = 0; i < B; i++) {
        rb.added_at[i] = p->reqs[req_ids[i]].added;
        rb.gen_at[i] = p->reqs[req_ids[i]].gen;
    }
    rb.pending = true;
    p->rb_next = (p->rb_next + 1) % sled_kvpool::READBACKS;
    return SLED_OK;
}

static int check_requests(sled_kvpool* p, int B, const int* req_ids, const char* who) {
    if (B < 1) SLED_FAIL(SLED_EINVAL, "%s: empty batch", who);
    std::vector<char> seen(p->max_requests, 0);
    for (int i = 0; i < B; i++) {
        int r = req_ids[i];
        if (r < 0 || r >= p->max_requests || !p->reqs[r].open) SLED_FAIL(SLED_EINVAL, "%s: request %d is not open", who, r);
        if (seen[r]) SLED_FAIL(SLED_EINVAL, "%s: request %d appears twice", who, r);
        seen[r] = 1;
    }
    return SLED_OK;
}

// make sure request r owns pages for `tokens` tokens
static int ensure_pages(sled_kvpool* p, int r, int tokens) {
    sled_request& rq = p->reqs[r];
    const int need = ceil_div(tokens, 16);
    while ((int)rq.pages.size() < need) {
        if (p->free_pages.empty()) SLED_FAIL(SLED_ENOMEM, "page pool exhausted (%lld pages)", (long long)p->n_pages);
        rq.pages.push_back(p->free_pages.back());
        p->free_pages.pop_back();
    }
    return SLED_OK;
}

extern "C" int sled_kvpool_lengths(sled_kvpool* p, int B, const int* req_ids, int* lens, void* stream) {
    if (!p || !req_ids || !lens) SLED_FAIL(SLED_EINVAL, "sled_kvpool_lengths: null argument");
    int rc = check_requests(p, B, req_ids, "sled_kvpool_lengths");
    if (rc != SLED_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    SLED_HIP(hipStreamSynchronize(st));
    poll_readbacks(p);
    std::vector<int32_t> all(p->max_requests);
    SLED_HIP(hipMemcpy(all.data(), p->len_dev, all.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
    for (int i = 0; i < B; i++) {
        sled_request& rq = p->reqs[req_ids[i]];
        lens[i] = rq.fresh ? 0 : all[req_ids[i]];   // a request nothing has touched yet is empty whatever the slot held
        rq.len_ub = lens[i];
        trim_pages(p, rq);   // rows staged by a verify that is not committed yet keep their pages
    }
    return SLED_OK;
}

extern "C" int sled_kv_append(sled_kvpool* p, int B, const int* req_ids, const int* n_tokens, const void* const* k_src,
                              const void* const* v_src, const int32_t* accept_len, void* stream) {
    if (!p || !req_ids) SLED_FAIL(SLED_EINVAL, "sled_kv_append: null argument");
    int rc = check_requests(p, B, req_ids, "sled_kv_append");
    if (rc != SLED_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const sled_model* m = p->m;
    poll_readbacks(p);
    if (accept_len) {
        // commit what the last verify staged
        for (int i = 0; i < B; i++)
            if (std::find(p->last_batch.begin(), p->last_batch.end(), req_ids[i]) == p->last_batch.end() ||
                p->reqs[req_ids[i]].staged < 0)
                SLED_FAIL(SLED_ESTATE, "sled_kv_append: request %d has nothing staged by the last verify", req_ids[i]);
        sled_stage_slot* sl;
        if ((rc = stage_acquire(p, B, &sl)) != SLED_OK) return rc;
        for (int i = 0; i < B; i++) sl->host[i] = req_ids[i];
        SLED_HIP(hipMemcpyAsync(sl->dev, sl->host, B * sizeof(int32_t), hipMemcpyHostToDevice, st));
        if ((rc = sled_launch_len_add(p->len_dev, sl->dev, nullptr, accept_len, B, st)) != SLED_OK) return rc;
        if ((rc = stage_release(sl, st)) != SLED_OK) return rc;
        for (int i = 0; i < B; i++) {
            sled_request& rq = p->reqs[req_ids[i]];
            rq.len_ub += rq.staged;  // upper bound: every staged row may have been accepted ...
            rq.added += rq.staged;
            rq.staged = -1;
            p->last_batch.erase(std::remove(p->last_batch.begin(), p->last_batch.end(), req_ids[i]), p->last_batch.end());
        }
        // ... and the exact lengths follow behind the commit, without anybody waiting for them
        return enqueue_readback(p, B, req_ids, st);
    }
    if (!n_tokens || !k_src || !v_src) SLED_FAIL(SLED_EINVAL, "sled_kv_append: null argument");
    if ((rc = reset_fresh_lengths(p, B, req_ids, st)) != SLED_OK) return rc;
    size_t need = 2 * (size_t)B;
    for (int i = 0; i < B; i++) {
        if (n_tokens[i] < 0 || (n_tokens[i] > 0 && (!k_src[i] || !v_src[i])))
            SLED_FAIL(SLED_EINVAL, "sled_kv_append: bad entry %d", i);
        if ((rc = ensure_pages(p, req_ids[i], p->reqs[req_ids[i]].len_ub + n_tokens[i])) != SLED_OK) return rc;
        need += p->reqs[req_ids[i]].pages.size();
    }
    sled_stage_slot* sl;
    if ((rc = stage_acquire(p, need, &sl)) != SLED_OK) return rc;
    size_t off = 2 * (size_t)B;
    std::vector<size_t> page_off(B);
    for (int i = 0; i < B; i++) {
        sl->host[i] = req_ids[i];
        sl->host[B + i] = n_tokens[i];
        page_off[i] = off;
        for (int pg : p->reqs[req_ids[i]].pages) sl->host[off++] = pg;
    }
    SLED_HIP(hipMemcpyAsync(sl->dev, sl->host, off * sizeof(int32_t), hipMemcpyHostToDevice, st));
    for (int i = 0; i < B; i++) {
        if (n_tokens[i] == 0) continue;
        if ((rc = sled_launch_kv_ingest(m, p, k_src[i], v_src[i], n_tokens[i], req_ids[i], sl->dev + page_off[i], st)) != SLED_OK)
            return rc;
    }
    if ((rc = sled_launch_len_add(p->len_dev, sl->dev, sl->dev + B, nullptr, B, st)) != SLED_OK) return rc;
    if ((rc = stage_release(sl, st)) != SLED_OK) return rc;
    for (int i = 0; i < B; i++) {
        sled_request& rq = p->reqs[req_ids[i]];
        rq.len_ub += n_tokens[i];
        rq.added += n_tokens[i];
        rq.staged = -1;   // rows staged by an uncommitted verify are overwritten: nothing of this request is left to commit
    }
    return SLED_OK;
}

extern "C" int sled_kv_read(sled_kvpool* p, int req_id, int first_token, int n_tokens, void* k_dst, void* v_dst, void* stream) {
    if (!p || !k_dst || !v_dst) SLED_FAIL(SLED_EINVAL, "sled_kv_read: null argument");
    int rc = check_requests(p, 1, &req_id, "sled_kv_read");
    if (rc != SLED_OK) return rc;
    const sled_request& rq = p->reqs[req_id];
    if (first_token < 0 || n_tokens < 1 || (int64_t)first_token + n_tokens > (int64_t)rq.pages.size() * 16)
        SLED_FAIL(SLED_EINVAL, "sled_kv_read: positions %d .. %d lie outside the %zu pages of request %d", first_token,
                  first_token + n_tokens - 1, rq.pages.size(), req_id);
    hipStream_t st = static_cast<hipStream_t>(stream);
    sled_stage_slot* sl;
    if ((rc = stage_acquire(p, rq.pages.size(), &sl)) != SLED_OK) return rc;
    for (size_t i = 0; i < rq.pages.size(); i++) sl->host[i] = rq.pages[i];
    SLED_HIP(hipMemcpyAsync(sl->dev, sl->host, rq.pages.size() * sizeof(int32_t), hipMemcpyHostToDevice, st));
    if ((rc = sled_launch_kv_export(p->m, p, k_dst, v_dst, first_token, n_tokens, sl->dev, st)) != SLED_OK) return rc;
    return stage_release(sl, st);
}

// ------------------------------------------------------------------------------------------ verify
namespace {

struct ws_plan {
    size_t h, xa, xo, xf, q, x1, partial, cs, kvslot, plan, part_o, part_ml, arrive, total, T_alloc;
};

// Attention work list.  A work item is a run of pages of one (request, kv head), processed by one
// workgroup.  Workgroups are handed to the eight XCDs round robin in launch order and start as CUs become free, so
// the launch takes as long as the busiest CU: one long request left whole can hold the launch for several times the
// average (a 64-request mix with contexts of 128 to 8192 tokens: 512 pages in one item against 243 per CU).  The
// pages-per-item bound is therefore chosen by playing the launch through on the host for a handful of candidate
// bounds and taking the one that finishes first; each (request, kv head) then splits its pages evenly.
//   - at least 32 pages (eight rounds of the page loop) per item and at most eight items per (request, kv head):
//     beyond that the hand-over between the items of a pair -- the last one to arrive reads the others' states --
//     costs more than the extra workgroups save;
//   - at most ATTN_ROUNDS items per CU beyond one per pair (this bounds the workspace);
//   - an item costs its pages plus a fixed part (prologue, folds, output, and that a CU which works alone at the end
//     of a launch streams faster than one of 256), and a little more when its pair is split (stored state, arrival
//     counter).  The two constants were fitted on the 64-request mix, the 70B batch and the 16-request batch: 16/8,
//     32/12, 48/16, 64/16, 96/24 were tried; 48/16 and 64/16 did best on the mix, all but the first left the others alone.
constexpr int ATTN_CUS = 256, ATTN_XCDS = 8, ATTN_ROUNDS = 4;
constexpr int ATTN_ITEM_FIXED = 48, ATTN_ITEM_SPLIT = 16;   // in units of one page's streaming time
constexpr int SLED_FIXED_CHUNK_PAGES = 48;  // 768 tokens; divisible by 4, 3 and 2 page groups
int attn_item_cap(int B, int Hkv) { return ATTN_ROUNDS * ATTN_CUS * ((B * Hkv + ATTN_CUS - 1) / ATTN_CUS); }
int attn_chunk(int np, int tgt) { return ceil_div(np, ceil_div(np, tgt)); }   // even split of a block's pages
// when the last workgroup ends if the blocks, in the order given, are cut into items of at most tgt pages
int64_t attn_makespan(const std::vector<int>& np, const std::vector<int>& order, int Hkv, int tgt) {
    constexpr int PER = ATTN_CUS / ATTN_XCDS;
    // per XCD a min-heap of the times its CUs become free; workgroup k goes to XCD k % 8
    static thread_local std::vector<int64_t> heap;
    heap.assign((size_t)ATTN_CUS, 0);
    auto cmp = [](int64_t a, int64_t b) { return a > b; };
    int64_t k = 0, end = 0;
    for (int i : order) {
        const int n = np[i], chunk = attn_chunk(n, tgt), pieces = ceil_div(n, chunk);
        for (int g = 0; g < Hkv; g++)
            for (int p0 = 0; p0 < n; p0 += chunk, k++) {
                int64_t* h = heap.data() + (k % ATTN_XCDS) * PER;
                std::pop_heap(h, h + PER, cmp);
                h[PER - 1] += std::min(chunk, n - p0) + ATTN_ITEM_FIXED + (pieces > 1 ? ATTN_ITEM_SPLIT : 0);
                end = std::max(end, h[PER - 1]);
                std::push_heap(h, h + PER, cmp);
            }
    }
    return end;
}
int attn_pages_per_item(const std::vector<int>& np, const std::vector<int>& order, int Hkv) {
    int longest = 1;
    for (int n : np) longest = std::max(longest, n);
    const int base = ATTN_CUS * (((int)np.size() * Hkv + ATTN_CUS - 1) / ATTN_CUS);
    const int lo = std::min(longest, std::max(32, ceil_div(longest, 8)));
    auto items = [&](int tgt) {
        int64_t k = 0;
        for (int n : np) k += (int64_t)Hkv * ceil_div(n, tgt);
        return k;
    };
    // candidates: the smallest bounds that give at most 1, 2, .. ATTN_ROUNDS items per CU (whole rounds of workgroups
    // of similar size), and a coarse geometric ladder between the limits
    int cand[ATTN_ROUNDS + 16], n_cand = 0;
    for (int c = 1; c <= ATTN_ROUNDS; c++) {
        int a = lo, b = longest;   // items() does not grow with the bound
        while (a < b) {
            const int mid = (a + b) / 2;
            if (items(mid) <= (int64_t)c * base) b = mid;
            else a = mid + 1;
        }
        cand[n_cand++] = a;
    }
    for (int tgt = lo; n_cand < ATTN_ROUNDS + 15; tgt += std::max(8, tgt / 3)) {
        cand[n_cand++] = std::min(tgt, longest);
        if (tgt >= longest) break;
    }
    int best = longest;
    int64_t best_end = -1;
    for (int c = 0; c < n_cand; c++) {
        if (items(cand[c]) > attn_item_cap((int)np.size(), Hkv)) continue;
        const int64_t end = attn_makespan(np, order, Hkv, cand[c]);
        if (best_end < 0 || end < best_end || (end == best_end && cand[c] > best)) {   // ties: fewer items
            best_end = end;
            best = cand[c];
        }
    }
    return best;
}

ws_plan plan_workspace(const sled_model* m, int T, int64_t n_work, int QT) {
    const sled_shape& s = m->s;
    const size_t T_alloc = align_up(T + 64, 128), T_pad = align_up(T, 32);  // row blocks of the GEMMs may overhang
    const size_t d = s.d_model, F = s.d_ffn, HD = (size_t)s.n_q_heads * s.head_dim;
    const size_t planes = s.dtype == SLED_BF16 ? 2 : 1;  // bf16 models keep activations as hi + lo
    ws_plan w;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off += align_up(bytes, 256);
        return o;
    };
    w.T_alloc = T_alloc;
    w.h = take(T_alloc * d * sizeof(float));
    w.xa = take(planes * T_alloc * d * m->elem);
    w.xo = take(planes * T_alloc * HD * m->elem);
    w.xf = take(planes * T_alloc * F * m->elem);
    w.q = take(planes * T_alloc * HD * m->elem);
    w.x1 = take(planes * 32 * d * m->elem);  // one 32-row tile: the single row whose logits a prompt asks for
    size_t part = 0;
    part = std::max(part, (size_t)sled_gemm_make_plan(m, m->n_qkv, s.d_model, false).cap * T_pad * m->n_qkv);
    part = std::max(part, (size_t)sled_gemm_make_plan(m, s.d_model, (int)HD, false).cap * T_pad * d);
    part = std::max(part, (size_t)sled_gemm_make_plan(m, s.d_model, s.d_ffn, false).cap * T_pad * d);
    part = std::max(part, (size_t)sled_gemm_make_plan(m, 2 * s.d_ffn, s.d_model, false).split * T_pad * 2 * F);
    w.partial = take(part * sizeof(float));
    w.cs = take((size_t)T * s.head_dim * sizeof(float));
    w.kvslot = take((size_t)T * sizeof(int32_t));
    w.plan = take((size_t)(n_work + 1) * 12 * sizeof(int32_t));   // one record per attention work item
    w.part_o = take((size_t)n_work * QT * 16 * 128 * sizeof(float));
    w.part_ml = take((size_t)n_work * 2 * QT * 16 * sizeof(float));
    w.arrive = take((size_t)(n_work + 1) * sizeof(int32_t));  // one counter per (request, kv head): at most n_work
    w.total = off;
    return w;
}

// upper bound of the attention work list
int max_work_items(const sled_model* m, int B, int64_t ctx_tokens) {
    const int balanced = attn_item_cap(B, m->s.n_kv_heads) + B * m->s.n_kv_heads;
    if (!m->batch_invariant) return balanced;
    // fixed runs of pages: one item per started run of every block and kv head
    const int64_t runs = ctx_tokens / (16 * SLED_FIXED_CHUNK_PAGES) + B;
    return (int)std::max<int64_t>(balanced, runs * m->s.n_kv_heads);
}

}  // namespace

extern "C" int sled_attention_partition(int n_kv_heads, int B, const int* n_pages, int* pages_per_item, int* n_items) {
    if (n_kv_heads < 1 || B < 1 || !n_pages || !pages_per_item || !n_items) SLED_FAIL(SLED_EINVAL, "sled_attention_partition: bad argument");
    std::vector<int> np(n_pages, n_pages + B), order(B);
    for (int i = 0; i < B; i++) {
        if (np[i] < 1) SLED_FAIL(SLED_EINVAL, "sled_attention_partition: request %d holds no page", i);
        order[i] = i;
    }
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return np[a] > np[b]; });
    const int tgt = attn_pages_per_item(np, order, n_kv_heads);
    int64_t items = 0;
    for (int n : np) items += (int64_t)n_kv_heads * ceil_div(n, attn_chunk(n, tgt));
    *pages_per_item = tgt;
    *n_items = (int)items;
    return SLED_OK;
}

extern "C" size_t sled_verify_workspace_bytes(const sled_model* m, int B_max, int T_max, int64_t ctx_tokens_max) {
    if (!m || B_max < 1 || T_max < 1 || ctx_tokens_max < 0) return 0;
    const int G = m->s.n_q_heads / m->s.n_kv_heads;
    const int QT = ceil_div(G * (m->s.k_max + 1), 16);
    size_t worst = 0;
    // the split-K choice depends on T only through nothing today, but take the maximum over the
    // padded sizes anyway so that the bound holds for every T <= T_max
    worst = plan_workspace(m, T_max, max_work_items(m, B_max, ctx_tokens_max), QT).total;
    return worst + 256;
}

namespace {

// One row block of a step: `rows` consecutive tokens of request `req`, the first of them `pos0` positions behind
// the request's committed length.  A verification request is one block (pos0 = 0, rows = k + 1); a prompt is cut
// into blocks of at most k_max + 1 rows that follow one another.
struct step_entry {
    int req, pos0, rows;
};

// The forward pass over the packed rows of `ent` on top of the cached contexts: new K/V go to the requests' pages
// (nothing is committed here), and the logits of all rows go to logits_all [T, vocab], or those of the single row
// one_row to logits_one [vocab], or nowhere.
int run_forward(sled_model* m, sled_kvpool* p, const std::vector<step_entry>& ent, const int32_t* tokens, float* logits_all,
                int one_row, float* logits_one, void* workspace, size_t workspace_bytes, hipStream_t st, const char* who) {
    const sled_shape& s = m->s;
    const int B = (int)ent.size();
    const int Hkv = s.n_kv_heads, G = s.n_q_heads / Hkv;
    int rc;
    int T = 0, nmax = 0;
    for (const step_entry& e : ent) {
        T += e.rows;
        nmax = std::max(nmax, e.rows);
    }
    // pages for the new tokens, attention work list
    int64_t total_pages = 0;
    std::vector<int> np_all(B);
    for (int i = 0; i < B; i++) {
        const sled_request& rq = p->reqs[ent[i].req];
        const int reach = rq.len_ub + ent[i].pos0 + ent[i].rows;  // upper bound of the last position + 1
        if ((rc = ensure_pages(p, ent[i].req, reach)) != SLED_OK) return rc;
        np_all[i] = ceil_div(reach, 16);
        total_pages += np_all[i];
    }
    // Pages per attention work item.  Normally whatever spreads this batch evenly over the CUs; for a
    // batch-invariant model a fixed run of pages, so that the keys of a request are always summed in the same
    // groups (a multiple of every page-group count the kernel uses).
    // Blocks with the most pages first: what is left for the end of the launch is then small.  (Batch-invariant:
    // the order of the batch, nothing may depend on the other requests.)
    std::vector<int> order(B);
    for (int i = 0; i < B; i++) order[i] = i;
    if (!m->batch_invariant) std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return np_all[a] > np_all[b]; });
    const int tgt = m->batch_invariant ? 0 : attn_pages_per_item(np_all, order, Hkv);
    std::vector<int32_t> work;
    std::vector<int32_t> cu_work(2 * B * Hkv);   // first and end item of (block, kv head), by block and head
    for (int i : order) {
        const int np = np_all[i];
        const int chunk = m->batch_invariant ? SLED_FIXED_CHUNK_PAGES : attn_chunk(np, tgt);
        for (int g = 0; g < Hkv; g++) {
            cu_work[2 * (i * Hkv + g)] = (int)(work.size() / 4);
            for (int p0 = 0; p0 < np; p0 += chunk) {
                work.push_back(i);
                work.push_back(g);
                work.push_back(p0);
                work.push_back(std::min(chunk, np - p0));
            }
            cu_work[2 * (i * Hkv + g) + 1] = (int)(work.size() / 4);
        }
    }
    const int n_work = (int)(work.size() / 4);
    // query tiles follow the longest block of the batch -- or, batch-invariant, of the model: the tile count sets
    // the number of page groups a workgroup splits its pages over
    const int QT = std::max(1, ceil_div(G * (m->batch_invariant ? s.k_max + 1 : nmax), 16));
    const ws_plan wp = plan_workspace(m, T, n_work, QT);
    if (wp.total > workspace_bytes) SLED_FAIL(SLED_EINVAL, "%s: workspace of %zu bytes, %zu needed", who, workspace_bytes, wp.total);

    // metadata blob
    const size_t n_meta = 3 * (size_t)B + 2 * ((size_t)B + 1) + 2 * (size_t)T + (size_t)total_pages + work.size() + cu_work.size();
    sled_stage_slot* sl;
    if ((rc = stage_acquire(p, n_meta, &sl)) != SLED_OK) return rc;
    int32_t* hp = sl->host;
    size_t o_req = 0, o_k = o_req + B, o_p0 = o_k + B, o_cur = o_p0 + B, o_cup = o_cur + B + 1, o_rr = o_cup + B + 1,
           o_rj = o_rr + T, o_pg = o_rj + T, o_wk = o_pg + total_pages, o_cw = o_wk + work.size();
    int row = 0, pg = 0;
    for (int i = 0; i < B; i++) {
        const sled_request& rq = p->reqs[ent[i].req];
        hp[o_req + i] = ent[i].req;
        hp[o_k + i] = ent[i].rows - 1;
        hp[o_p0 + i] = ent[i].pos0;
        hp[o_cur + i] = row;
        hp[o_cup + i] = pg;
        for (int j = 0; j < ent[i].rows; j++) {
            hp[o_rr + row] = i;
            hp[o_rj + row] = j;
            row++;
        }
        for (int q = 0; q < np_all[i]; q++) hp[o_pg + pg++] = rq.pages[q];
    }
    hp[o_cur + B] = row;
    hp[o_cup + B] = pg;
    memcpy(hp + o_wk, work.data(), work.size() * sizeof(int32_t));
    memcpy(hp + o_cw, cu_work.data(), cu_work.size() * sizeof(int32_t));
    SLED_HIP(hipMemcpyAsync(sl->dev, hp, n_meta * sizeof(int32_t), hipMemcpyHostToDevice, st));
    sled_step_meta meta;
    meta.req_id = sl->dev + o_req;
    meta.k = sl->dev + o_k;
    meta.pos0 = sl->dev + o_p0;
    meta.cu_rows = sl->dev + o_cur;
    meta.cu_pages = sl->dev + o_cup;
    meta.row_req = sl->dev + o_rr;
    meta.row_j = sl->dev + o_rj;
    meta.pages = sl->dev + o_pg;
    meta.work = sl->dev + o_wk;
    meta.cu_work = sl->dev + o_cw;
    meta.B = B;
    meta.T = T;
    meta.n_work = n_work;

    char* ws = static_cast<char*>(workspace);
    float* h = reinterpret_cast<float*>(ws + wp.h);
    void* xa = ws + wp.xa;
    void* xo = ws + wp.xo;
    void* xf = ws + wp.xf;
    void* qb = ws + wp.q;
    void* x1 = ws + wp.x1;
    float* partial = reinterpret_cast<float*>(ws + wp.partial);
    float* cs = reinterpret_cast<float*>(ws + wp.cs);
    int32_t* kvslot = reinterpret_cast<int32_t*>(ws + wp.kvslot);
    int32_t* plan = reinterpret_cast<int32_t*>(ws + wp.plan);
    float* part_o = reinterpret_cast<float*>(ws + wp.part_o);
    float* part_ml = reinterpret_cast<float*>(ws + wp.part_ml);
    int32_t* arrive = reinterpret_cast<int32_t*>(ws + wp.arrive);
    const int T_pad = (int)align_up(T, 32);
    const int d = s.d_model, F = s.d_ffn, HD = s.n_q_heads * s.head_dim;
    const bool bf = s.dtype == SLED_BF16;
    // distance between the hi and lo planes of each activation buffer (bf16 models)
    const size_t pl_d = bf ? wp.T_alloc * (size_t)d : 0, pl_hd = bf ? wp.T_alloc * (size_t)HD : 0,
                 pl_f = bf ? wp.T_alloc * (size_t)F : 0;
    // K slices: the model's plan (which sized the workspace), thinned out for this step's number of rows
    const sled_gemm_plan g_qkv = sled_gemm_plan_rows(m, sled_gemm_make_plan(m, m->n_qkv, d, false), m->n_qkv, d, T_pad),
                         g_o = sled_gemm_plan_rows(m, sled_gemm_make_plan(m, d, HD, false), d, HD, T_pad),
                         g_dn = sled_gemm_plan_rows(m, sled_gemm_make_plan(m, d, F, false), d, F, T_pad),
                         g_lm = sled_gemm_make_plan(m, s.vocab, d, true);
    // gate/up applies SwiGLU in its epilogue when it runs unsplit; otherwise (and for fp32 models) a row
    // kernel reduces the K slices and applies it
    sled_gemm_plan g_gu = sled_gemm_make_plan(m, 2 * F, d, false);
    const bool gu_fused = bf && g_gu.split == 1;
    // The attention kernel takes the QKV projection's partial sums itself (sum over K slices, rotary, K/V write) when
    // every block is a request of its own at offset 0, i.e. in a verification step.  The blocks of a prompt slice read
    // keys that other blocks of the same slice write, so there all new K/V must be in the cache before attention
    // starts: the stand-alone row kernel does it.
    bool qkv_fused = bf;
    for (const step_entry& e : ent) qkv_fused = qkv_fused && e.pos0 == 0;
    if (qkv_fused) {
        std::vector<char> seen(p->max_requests, 0);
        for (const step_entry& e : ent) {
            if (seen[e.req]) qkv_fused = false;
            seen[e.req] = 1;
        }
    }

#define SLED_TRY(x)                        \
    do {                                   \
        if ((rc = (x)) != SLED_OK) return rc; \
    } while (0)
// a launch inside a timing scope of class c
#define SLED_RUN(c, x)                     \
    do {                                   \
        prof_scope _ps(m, (c), st);        \
        SLED_TRY(x);                       \
    } while (0)

    // arrival counters of the attention work items start at zero (each layer leaves them at zero)
    SLED_RUN(SLED_PROF_ROWS, sled_launch_fill_i32(arrive, 0, (size_t)B * Hkv, st));
    SLED_RUN(SLED_PROF_ROWS, sled_launch_rope_table(m, p, meta, cs, kvslot, st));
    if (bf) SLED_RUN(SLED_PROF_ROWS, sled_launch_attn_plan(m, p, meta, plan, st));
    SLED_RUN(SLED_PROF_ROWS, sled_launch_embed_norm(m, tokens, T, h, xa, pl_d, m->layers[0].g_attn, st));
    for (int l = 0; l < s.n_layers; l++) {
        const sled_layer_weights& w = m->layers[l];
        SLED_RUN(SLED_PROF_PROJ, sled_launch_gemm(m, xa, pl_d, w.w_qkv, w.s_qkv, T, T_pad, m->n_qkv, d, SLED_EPI_PARTIAL, g_qkv, partial, nullptr, 0, 0, st));
        if (qkv_fused) {
            SLED_RUN(SLED_PROF_ATTN, sled_launch_attention(m, p, meta, l, nullptr, 0, partial, g_qkv.split, T_pad, cs, kvslot, plan, part_o, part_ml, arrive, xo, pl_hd, QT, st));
        } else {
            SLED_RUN(SLED_PROF_ROWS, sled_launch_qkv_rope_store(m, p, T, l, partial, g_qkv.split, T_pad, cs, kvslot, qb, pl_hd, st));
            SLED_RUN(SLED_PROF_ATTN, sled_launch_attention(m, p, meta, l, qb, pl_hd, nullptr, 0, 0, nullptr, nullptr, plan, part_o, part_ml, arrive, xo, pl_hd, QT, st));
        }
        SLED_RUN(SLED_PROF_PROJ, sled_launch_gemm(m, xo, pl_hd, w.w_o, w.s_o, T, T_pad, d, HD, SLED_EPI_PARTIAL, g_o, partial, nullptr, 0, 0, st));
        SLED_RUN(SLED_PROF_ROWS, sled_launch_residual_norm(m, partial, g_o.split, T, T_pad, h, xa, pl_d, w.g_mlp, st));
        if (gu_fused) {
            SLED_RUN(SLED_PROF_PROJ, sled_launch_gemm(m, xa, pl_d, w.w_gu, w.s_gu, T, T_pad, 2 * F, d, SLED_EPI_SWIGLU, g_gu, nullptr, xf, pl_f, F, st));
        } else {
            SLED_RUN(SLED_PROF_PROJ, sled_launch_gemm(m, xa, pl_d, w.w_gu, w.s_gu, T, T_pad, 2 * F, d, SLED_EPI_PARTIAL, g_gu, partial, nullptr, 0, 0, st));
            SLED_RUN(SLED_PROF_ROWS, sled_launch_swiglu_reduce(m, partial, g_gu.split, T, T_pad, xf, pl_f, st));
        }
        SLED_RUN(SLED_PROF_PROJ, sled_launch_gemm(m, xf, pl_f, w.w_down, w.s_down, T, T_pad, d, F, SLED_EPI_PARTIAL, g_dn, partial, nullptr, 0, 0, st));
        const float* next_gain = (l + 1 < s.n_layers) ? m->layers[l + 1].g_attn : m->g_final;
        SLED_RUN(SLED_PROF_ROWS, sled_launch_residual_norm(m, partial, g_dn.split, T, T_pad, h, xa, pl_d, next_gain, st));
    }
    if (logits_all) {
        SLED_RUN(SLED_PROF_PROJ, sled_launch_gemm(m, xa, pl_d, m->lm_head, m->s_lm, T, T_pad, s.vocab, d, SLED_EPI_STORE, g_lm, logits_all, nullptr, 0, 0, st));
    } else if (one_row >= 0 && logits_one) {
        // the LM head over one row: that row becomes row 0 of a one-tile activation block
        const size_t pl_1 = bf ? (size_t)32 * d : 0;
        SLED_RUN(SLED_PROF_ROWS, sled_launch_copy_act_row(m, xa, pl_d, one_row, x1, pl_1, d, st));
        SLED_RUN(SLED_PROF_PROJ, sled_launch_gemm(m, x1, pl_1, m->lm_head, m->s_lm, 1, 32, s.vocab, d, SLED_EPI_STORE, g_lm, logits_one, nullptr, 0, 0, st));
    }
    SLED_TRY(stage_release(sl, st));
#undef SLED_RUN
#undef SLED_TRY
    return SLED_OK;
}

}  // namespace

extern "C" int sled_verify_batch(sled_model* m, sled_kvpool* p, int B, const int* req_ids, const int* k,
                                 const int32_t* tokens, float* logits, void* workspace, size_t workspace_bytes,
                                 void* stream) {
    if (!m || !p || !req_ids || !k || !tokens || !logits || !workspace) SLED_FAIL(SLED_EINVAL, "sled_verify_batch: null argument");
    if (p->m != m) SLED_FAIL(SLED_EINVAL, "sled_verify_batch: pool belongs to another model");
    if (reinterpret_cast<uintptr_t>(workspace) % 256) SLED_FAIL(SLED_EINVAL, "sled_verify_batch: workspace must be 256-byte aligned");
    int rc = check_requests(p, B, req_ids, "sled_verify_batch");
    if (rc != SLED_OK) return rc;
    std::vector<step_entry> ent(B);
    for (int i = 0; i < B; i++) {
        if (k[i] < 0 || k[i] > m->s.k_max) SLED_FAIL(SLED_EINVAL, "sled_verify_batch: k[%d] = %d outside [0, %d]", i, k[i], m->s.k_max);
        ent[i] = step_entry{req_ids[i], 0, k[i] + 1};
    }
    poll_readbacks(p);
    if ((rc = reset_fresh_lengths(p, B, req_ids, static_cast<hipStream_t>(stream))) != SLED_OK) return rc;
    rc = run_forward(m, p, ent, tokens, logits, -1, nullptr, workspace, workspace_bytes, static_cast<hipStream_t>(stream),
                     "sled_verify_batch");
    if (rc != SLED_OK) return rc;
    // what an earlier verify staged for requests that are not in this batch stays staged, but only the last batch
    // can be committed
    for (int r : p->last_batch) p->reqs[r].staged = -1;
    for (int i = 0; i < B; i++) p->reqs[req_ids[i]].staged = k[i] + 1;
    p->last_batch.assign(req_ids, req_ids + B);
    return SLED_OK;
}

extern "C" int sled_prefill(sled_model* m, sled_kvpool* p, int req_id, int n_tokens, const int32_t* tokens, float* logits_last,
                            void* workspace, size_t workspace_bytes, void* stream) {
    if (!m || !p || !tokens || !workspace) SLED_FAIL(SLED_EINVAL, "sled_prefill: null argument");
    if (p->m != m) SLED_FAIL(SLED_EINVAL, "sled_prefill: pool belongs to another model");
    if (reinterpret_cast<uintptr_t>(workspace) % 256) SLED_FAIL(SLED_EINVAL, "sled_prefill: workspace must be 256-byte aligned");
    if (n_tokens < 1) SLED_FAIL(SLED_EINVAL, "sled_prefill: n_tokens = %d", n_tokens);
    int rc = check_requests(p, 1, &req_id, "sled_prefill");
    if (rc != SLED_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const sled_shape& s = m->s;
    // Rows of one block.  Every block reads all keys before it, so longer blocks mean fewer passes over the cache:
    // a prompt takes the most rows the attention kernel's five query tiles hold (80 stacked (head, row) pairs per kv
    // head: 20 tokens at four query heads per kv head), not the k_max + 1 of a verification request.  A batch-invariant
    // model keeps k_max + 1, the block its fixed summation order is defined for.
    const int G = s.n_q_heads / s.n_kv_heads;
    const int64_t reach = (int64_t)p->reqs[req_id].len_ub + n_tokens;  // every block of a slice may see that many keys
    int per = s.k_max + 1, QT = ceil_div(G * per, 16);
    auto fits_with = [&](int rows_per_block, int tiles, int blocks) {
        return plan_workspace(m, blocks * rows_per_block, max_work_items(m, blocks, blocks * reach), tiles).total <= workspace_bytes;
    };
    auto most_blocks = [&](int rows_per_block, int tiles) {   // blocks of a slice the workspace holds (0: not even one)
        if (!fits_with(rows_per_block, tiles, 1)) return 0;
        int lo = 1, hi = ceil_div(n_tokens, rows_per_block);
        while (lo < hi) {
            const int mid = (lo + hi + 1) / 2;
            if (fits_with(rows_per_block, tiles, mid)) lo = mid;
            else hi = mid - 1;
        }
        return lo;
    };
    if (s.dtype == SLED_BF16 && !m->batch_invariant) {
        // long blocks only where they still leave a work item for every CU: a small workspace (short slices) is
        // better served by many short blocks (measured: 126-row slices 15 % slower with 20-row blocks)
        const int big = std::max(per, 80 / G), big_qt = ceil_div(G * big, 16);
        if (big > per && (int64_t)most_blocks(big, big_qt) * s.n_kv_heads >= 256) {
            per = big;
            QT = big_qt;
        }
    }
    // the largest number of blocks per step that the workspace holds
    auto fits = [&](int blocks) { return fits_with(per, QT, blocks); };
    if (!fits(1)) SLED_FAIL(SLED_EINVAL, "sled_prefill: workspace of %zu bytes is too small for one block of %d rows", workspace_bytes, per);
    int lo = 1, hi = ceil_div(n_tokens, per);
    while (lo < hi) {  // fits(lo) holds
        const int mid = (lo + hi + 1) / 2;
        if (fits(mid)) lo = mid;
        else hi = mid - 1;
    }
    const int blocks_per_step = lo;
    sled_request& rq = p->reqs[req_id];
    poll_readbacks(p);
    if ((rc = reset_fresh_lengths(p, 1, &req_id, st)) != SLED_OK) return rc;
    // rows staged for THIS request by an earlier verify are overwritten, so it has nothing left to commit; the other
    // requests of that verify keep their staged rows and their commit stays valid
    rq.staged = -1;
    for (int done = 0; done < n_tokens;) {
        const int rows = std::min(n_tokens - done, blocks_per_step * per);
        std::vector<step_entry> ent;
        for (int r = 0; r < rows; r += per) ent.push_back(step_entry{req_id, r, std::min(per, rows - r)});
        const bool last = done + rows == n_tokens;
        rc = run_forward(m, p, ent, tokens + done, nullptr, (last && logits_last) ? rows - 1 : -1, logits_last, workspace,
                         workspace_bytes, st, "sled_prefill");
        if (rc != SLED_OK) return rc;
        // commit the slice: L += rows, in stream order before the next slice reads L
        sled_stage_slot* sl;
        if ((rc = stage_acquire(p, 2, &sl)) != SLED_OK) return rc;
        sl->host[0] = req_id;
        sl->host[1] = rows;
        SLED_HIP(hipMemcpyAsync(sl->dev, sl->host, 2 * sizeof(int32_t), hipMemcpyHostToDevice, st));
        if ((rc = sled_launch_len_add(p->len_dev, sl->dev, sl->dev + 1, nullptr, 1, st)) != SLED_OK) return rc;
        if ((rc = stage_release(sl, st)) != SLED_OK) return rc;
        rq.len_ub += rows;
        rq.added += rows;
        done += rows;
    }
    return SLED_OK;
}

// ------------------------------------------------------------------------------------------ accept
extern "C" size_t sled_accept_workspace_bytes(int B, int T, int vocab) {
    if (B < 1 || T < 1 || vocab < 2) return 0;
    return sled_accept_ws_bytes(B, T, 16) + 256;
}

namespace {

// checks shared by the two acceptance entry points; on success *T_out = packed rows, *nd_out = drafts
int accept_checks(const char* who, int mode, int B, const int* k, int vocab, float temperature, const void* logits,
                  const void* tokens, const void* accept_len, const void* out_token, void* workspace, size_t workspace_bytes,
                  int* T_out, int* nd_out) {
    if (!k || !logits || !tokens || !accept_len || !out_token || !workspace) SLED_FAIL(SLED_EINVAL, "%s: null argument", who);
    if (mode != SLED_GREEDY && mode != SLED_SAMPLE) SLED_FAIL(SLED_EINVAL, "%s: unknown mode %d", who, mode);
    if (B < 1 || B > 1024) SLED_FAIL(SLED_EINVAL, "%s: batch size %d outside [1, 1024]", who, B);
    if (vocab < 2 || vocab > 2000000) SLED_FAIL(SLED_EINVAL, "%s: vocab %d unsupported", who, vocab);
    if (!(temperature > 0.f)) SLED_FAIL(SLED_EINVAL, "%s: temperature must be positive", who);
    int T = 0, nd = 0;
    for (int i = 0; i < B; i++) {
        if (k[i] < 0 || k[i] > 255) SLED_FAIL(SLED_EINVAL, "%s: k[%d] = %d outside [0, 255]", who, i, k[i]);
        T += k[i] + 1;
        nd += k[i];
    }
    if (reinterpret_cast<uintptr_t>(workspace) % 256) SLED_FAIL(SLED_EINVAL, "%s: workspace must be 256-byte aligned", who);
    const size_t need = sled_accept_ws_bytes(B, T, sled_accept_pick_split(T, vocab));
    if (need > workspace_bytes) SLED_FAIL(SLED_EINVAL, "%s: workspace of %zu bytes, %zu needed", who, workspace_bytes, need);
    *T_out = T;
    *nd_out = nd;
    return SLED_OK;
}

}  // namespace

extern "C" int sled_accept(int mode, int B, const int* k, int vocab, float temperature, const float* logits,
                           const int32_t* tokens, const float* draft_q, const float* u_acc, const float* u_smp,
                           int32_t* accept_len, int32_t* out_token, void* workspace, size_t workspace_bytes,
                           void* stream) {
    int T, nd;
    int rc = accept_checks("sled_accept", mode, B, k, vocab, temperature, logits, tokens, accept_len, out_token, workspace,
                           workspace_bytes, &T, &nd);
    if (rc != SLED_OK) return rc;
    if (mode == SLED_SAMPLE && (!u_smp || (nd > 0 && (!draft_q || !u_acc))))
        SLED_FAIL(SLED_EINVAL, "sled_accept: sampling needs draft_q, u_acc and u_smp");
    return sled_launch_accept(mode, B, T, k, vocab, temperature, logits, tokens, draft_q, nullptr, nullptr, nullptr, 0, u_acc,
                              u_smp, accept_len, out_token, workspace, static_cast<hipStream_t>(stream));
}

extern "C" int sled_accept_sparse(int B, const int* k, int vocab, float temperature, const float* logits, const int32_t* tokens,
                                  int q_m, const int32_t* q_ids, const float* q_probs, const float* q_rest, const float* u_acc,
                                  const float* u_smp,
                                  int32_t* accept_len, int32_t* out_token, void* workspace, size_t workspace_bytes,
                                  void* stream) {
    int T, nd;
    int rc = accept_checks("sled_accept_sparse", SLED_SAMPLE, B, k, vocab, temperature, logits, tokens, accept_len, out_token,
                           workspace, workspace_bytes, &T, &nd);
    if (rc != SLED_OK) return rc;
    if (q_m < 1 || q_m > 1024) SLED_FAIL(SLED_EINVAL, "sled_accept_sparse: %d entries per draft outside [1, 1024]", q_m);
    if (!u_smp || (nd > 0 && (!q_ids || !q_probs || !u_acc)))
        SLED_FAIL(SLED_EINVAL, "sled_accept_sparse: needs q_ids, q_probs, u_acc and u_smp");
    return sled_launch_accept(SLED_SAMPLE, B, T, k, vocab, temperature, logits, tokens, nullptr, q_ids, q_probs, q_rest, q_m, u_acc,
                              u_smp, accept_len, out_token, workspace, static_cast<hipStream_t>(stream));
}

extern "C" int sled_row_confidence(int T, int vocab, float temperature, const float* logits, float* conf, int32_t* top,
                                   void* workspace, size_t workspace_bytes, void* stream) {
    if (!logits || !conf || !workspace) SLED_FAIL(SLED_EINVAL, "sled_row_confidence: null argument");
    if (T < 1 || T > (1 << 20)) SLED_FAIL(SLED_EINVAL, "sled_row_confidence: %d rows outside [1, 2^20]", T);
    if (vocab < 2 || vocab > 2000000) SLED_FAIL(SLED_EINVAL, "sled_row_confidence: vocab %d unsupported", vocab);
    if (!(temperature > 0.f)) SLED_FAIL(SLED_EINVAL, "sled_row_confidence: temperature must be positive");
    if (reinterpret_cast<uintptr_t>(workspace) % 256) SLED_FAIL(SLED_EINVAL, "sled_row_confidence: workspace must be 256-byte aligned");
    const size_t need = sled_accept_ws_bytes(1, T, sled_accept_pick_split(T, vocab));
    if (need > workspace_bytes) SLED_FAIL(SLED_EINVAL, "sled_row_confidence: workspace of %zu bytes, %zu needed", workspace_bytes, need);
    return sled_launch_row_confidence(T, vocab, temperature, logits, conf, top, workspace, static_cast<hipStream_t>(stream));
}
