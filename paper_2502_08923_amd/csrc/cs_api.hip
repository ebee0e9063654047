// C ABI of libcopyspec: handles, the verify pass, the whole step and the decode loops.
// Host logic only; every arithmetic step runs in the kernels of the other files.
#include <stdarg.h>
#include <stdlib.h>
#include <cmath>

#include <vector>

#include "cs_common.h"

// -------------------------------------------------------------------------------------
// errors
// -------------------------------------------------------------------------------------
static thread_local char g_err[512] = "";

void cs_set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

extern "C" const char* cs_last_error(void) { return g_err; }
extern "C" const char* cs_version(void) { return "copyspec-gfx950 0.1"; }

static thread_local int g_plain = 0;
extern "C" void cs_set_plain_kernels(int32_t on) { g_plain = on ? 1 : 0; }

// Rows of one prompt block.  With thousands of rows the projections of a block are compute-bound
// with few K splits and the block's attention fills the chip without splitting the token axis;
// measured at the 8B shape, a prompt goes in 65 % faster in 4096-row blocks than in 512-row
// blocks (2048: 4 % slower than 4096; 6144 and 8192: no faster).
#define CS_PROMPT_BLOCK_ROWS 4096
static thread_local int g_prompt_rows = 0;
extern "C" void cs_set_prompt_block_rows(int32_t rows) {
    g_prompt_rows = rows <= 0 ? 0 : (rows < 16 ? 16 : (rows > 8192 ? 8192 : rows));
}

// -------------------------------------------------------------------------------------
// instrumentation
// -------------------------------------------------------------------------------------
struct prof_slot { int cls; hipEvent_t a, b; };
static std::vector<prof_slot> g_prof;
static size_t g_prof_used = 0;
static int g_prof_mask = 0;

int cs_prof_begin(int cls, hipStream_t s) {
    if (!(g_prof_mask & cls)) return -1;
    if (g_prof_used == g_prof.size()) {
        if (g_prof.size() >= 200000) return -1;
        prof_slot ps;
        ps.cls = cls;
        if (hipEventCreate(&ps.a) != hipSuccess || hipEventCreate(&ps.b) != hipSuccess) return -1;
        g_prof.push_back(ps);
    }
    prof_slot& ps = g_prof[g_prof_used];
    ps.cls = cls;
    (void)hipEventRecord(ps.a, s);
    return (int)g_prof_used++;
}

void cs_prof_end(int slot, hipStream_t s) {
    if (slot >= 0) (void)hipEventRecord(g_prof[slot].b, s);
}

extern "C" void cs_profile_enable(int32_t mask) { g_prof_mask = mask; }
extern "C" void cs_profile_reset(void) {
    (void)hipDeviceSynchronize();
    g_prof_used = 0;
}
extern "C" int cs_profile_read(int32_t cls, double* total_ms, int64_t* launches) {
    CS_REQUIRE(total_ms && launches, CS_E_ARG, "cs_profile_read: NULL output");
    CS_HIP(hipDeviceSynchronize());
    double tot = 0.0;
    int64_t n = 0;
    for (size_t i = 0; i < g_prof_used; ++i) {
        if (g_prof[i].cls != cls) continue;
        float ms = 0.f;
        CS_HIP(hipEventElapsedTime(&ms, g_prof[i].a, g_prof[i].b));
        tot += ms;
        ++n;
    }
    *total_ms = tot;
    *launches = n;
    return CS_OK;
}

// -------------------------------------------------------------------------------------
// small kernels used only here
// -------------------------------------------------------------------------------------
// interleave gate and up rows in blocks of 16: dst row (f/16)*32 + 16*u + f%16
template <typename T>
__global__ void k_pack_gu(const T* __restrict__ wg, const T* __restrict__ wu, int F, int d,
                          T* __restrict__ dst) {
    const int row = blockIdx.x;               // destination row
    const int f = (row / 32) * 16 + row % 16;
    const T* __restrict__ src = ((row / 16) % 2 ? wu : wg) + (int64_t)f * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) dst[(int64_t)row * d + c] = src[c];
}

// V rows [KVH][n][hd] <-> cache [KVH][cap/128][hd][128] (cs_v_index)
template <typename T, int TO_CACHE>
__global__ void k_v_transpose(T* __restrict__ cache, T* __restrict__ rows, int64_t cap, int hd,
                              int64_t pos0, int64_t n) {
    const int g = blockIdx.y;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n * hd;
         idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t t = idx / hd;
        const int d = (int)(idx % hd);
        T* c = cache + (int64_t)g * hd * cap + cs_v_index(pos0 + t, d, hd);
        T* r = rows + ((int64_t)g * n + t) * hd + d;
        if (TO_CACHE) *c = *r; else *r = *c;
    }
}

__global__ void k_pending(const int32_t* __restrict__ hist, int64_t stride,
                          const int32_t* __restrict__ hist_len, int B, int32_t* __restrict__ pending) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    // (an empty history has no pending token: token 0 keeps the block well-formed)
    if (b < B) pending[b] = hist_len[b] >= 1 ? hist[(int64_t)b * stride + hist_len[b] - 1] : 0;
}

__global__ void k_add_i32(int32_t* p, int32_t v, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] += v;
}

__global__ void k_add_i32_vec(int32_t* p, const int32_t* __restrict__ v, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] += v[i];
}

// the tokens a step appended to each history: out[b][0 .. accepted[b]] (k+1 slots per stream)
__global__ void k_emitted(const int32_t* __restrict__ hist, int64_t stride,
                          const int32_t* __restrict__ hist_len, const int32_t* __restrict__ accepted,
                          int k, int32_t* __restrict__ out) {
    const int b = blockIdx.x;
    const int got = accepted[b] + 1;
    const int32_t* __restrict__ h = hist + (int64_t)b * stride + hist_len[b] - got;
    for (int i = threadIdx.x; i < got; i += blockDim.x) out[b * (k + 1) + i] = h[i];
}

__global__ void k_sum_parts(const float* __restrict__ part, int nparts, int64_t n,
                            float* __restrict__ y) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x) {
        float a = 0.f;
        for (int p = 0; p < nparts; ++p) a += part[p * n + i];
        y[i] = a;
    }
}

// -------------------------------------------------------------------------------------
// model
// -------------------------------------------------------------------------------------
static int dev_alloc(void** p, size_t bytes) {
    *p = nullptr;
    CS_HIP(hipMalloc(p, bytes ? bytes : 16));
    return CS_OK;
}
#define DEV_ALLOC(ptr, bytes) CS_TRY(dev_alloc((void**)&(ptr), (bytes)))

static void model_free(cs_model* m) {
    if (!m) return;
    void* ptrs[] = {m->embed, m->lm_head, m->final_norm, m->x, m->xn, m->q, m->gu, m->act,
                    m->logits, m->part, m->attn_part, m->rope, m->tok, m->am_val_idx,
                    m->row_argmax, m->draft, m->draft_len, m->match_pos, m->pending, m->range_flags,
                    m->rope_inv_freq};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    if (m->layers) {
        for (int l = 0; l < m->cfg.n_layers; ++l) {
            cs_layer_dev& L = m->layers[l];
            void* lp[] = {L.wqkv, L.wo, L.wgu, L.wd, L.norm1, L.norm2, L.bqkv};
            for (void* p : lp)
                if (p) (void)hipFree(p);
        }
        free(m->layers);
    }
    free(m->layer_loaded);
    free(m);
}

// the float16 matrix cores cannot hold every bfloat16 weight: checked after every load
static int weight_range_check(cs_model* m) {
    CS_HIP(hipDeviceSynchronize());
    if (!m->fast) return CS_OK;
    int32_t flags = 0;
    CS_HIP(hipMemcpy(&flags, m->range_flags, 4, hipMemcpyDeviceToHost));
    CS_REQUIRE(!(flags & CS_RANGE_WEIGHT), CS_E_UNSUPPORTED,
               "a projection weight is not finite or exceeds 65504 in magnitude: the float16 matrix "
               "cores cannot hold it (cs_set_plain_kernels(1) selects kernels without this limit)");
    return CS_OK;
}

// embedding, final norm gain and lm_head into the library's own storage
static int model_load_head(cs_model* m, const void* embed, const void* lm_head, const float* final_norm) {
    const cs_model_cfg& c = m->cfg;
    const size_t e = m->esz;
    const int d = c.d_model, V = c.vocab;
    CS_REQUIRE(embed && lm_head && final_norm, CS_E_ARG, "NULL weight pointer");
    CS_HIP(hipMemcpy(m->embed, embed, (size_t)V * d * e, hipMemcpyDeviceToDevice));
    CS_HIP(hipMemcpy(m->final_norm, final_norm, (size_t)d * 4, hipMemcpyDeviceToDevice));
    if (m->fast) CS_TRY(cs_tile_weights_launch(lm_head, nullptr, V, d, 0, V, 0, m->lm_head, m->range_flags, nullptr));
    else CS_HIP(hipMemcpy(m->lm_head, lm_head, (size_t)V * d * e, hipMemcpyDeviceToDevice));
    CS_TRY(weight_range_check(m));
    m->head_loaded = 1;
    return CS_OK;
}

// one layer's weights into the library's own storage (re-laid-out for the tuned kernels)
static int model_load_layer(cs_model* m, int l, const cs_layer_weights& s) {
    const cs_model_cfg& c = m->cfg;
    const size_t e = m->esz;
    const int d = c.d_model, hd = c.head_dim, H = c.n_heads, KVH = c.n_kv_heads, F = c.d_ff;
    const int nq = H * hd, nkv = KVH * hd, nqkv = nq + 2 * nkv;
    CS_REQUIRE(s.wq && s.wk && s.wv && s.wo && s.wg && s.wu && s.wd && s.norm1 && s.norm2,
               CS_E_ARG, "layer %d has a NULL weight pointer", l);
    cs_layer_dev& L = m->layers[l];
    char* qkv = (char*)L.wqkv;
    CS_HIP(hipMemcpy(L.norm1, s.norm1, (size_t)d * 4, hipMemcpyDeviceToDevice));
    CS_HIP(hipMemcpy(L.norm2, s.norm2, (size_t)d * 4, hipMemcpyDeviceToDevice));
    if (s.bq || s.bk || s.bv) {
        CS_REQUIRE(s.bq && s.bk && s.bv, CS_E_ARG, "layer %d: the q, k, v biases come all three or not at all", l);
        if (!L.bqkv) DEV_ALLOC(L.bqkv, (size_t)nqkv * 4);
        CS_HIP(hipMemcpy(L.bqkv, s.bq, (size_t)nq * 4, hipMemcpyDeviceToDevice));
        CS_HIP(hipMemcpy(L.bqkv + nq, s.bk, (size_t)nkv * 4, hipMemcpyDeviceToDevice));
        CS_HIP(hipMemcpy(L.bqkv + nq + nkv, s.bv, (size_t)nkv * 4, hipMemcpyDeviceToDevice));
    } else if (L.bqkv) {
        (void)hipFree(L.bqkv);
        L.bqkv = nullptr;
    }
    if (m->fast) {
        // the q, k and v blocks become row ranges of one tiled matrix
        CS_TRY(cs_tile_weights_launch(s.wq, nullptr, nq, d, 0, nqkv, 0, qkv, m->range_flags, nullptr));
        CS_TRY(cs_tile_weights_launch(s.wk, nullptr, nkv, d, 0, nqkv, nq, qkv, m->range_flags, nullptr));
        CS_TRY(cs_tile_weights_launch(s.wv, nullptr, nkv, d, 0, nqkv, nq + nkv, qkv, m->range_flags, nullptr));
        CS_TRY(cs_tile_weights_launch(s.wo, nullptr, d, nq, 0, d, 0, L.wo, m->range_flags, nullptr));
        CS_TRY(cs_tile_weights_launch(s.wg, s.wu, 2 * F, d, 1, 2 * F, 0, L.wgu, m->range_flags, nullptr));
        CS_TRY(cs_tile_weights_launch(s.wd, nullptr, d, F, 0, d, 0, L.wd, m->range_flags, nullptr));
    } else {
        CS_HIP(hipMemcpy(qkv, s.wq, (size_t)nq * d * e, hipMemcpyDeviceToDevice));
        CS_HIP(hipMemcpy(qkv + (size_t)nq * d * e, s.wk, (size_t)nkv * d * e, hipMemcpyDeviceToDevice));
        CS_HIP(hipMemcpy(qkv + (size_t)(nq + nkv) * d * e, s.wv, (size_t)nkv * d * e,
                         hipMemcpyDeviceToDevice));
        CS_HIP(hipMemcpy(L.wo, s.wo, (size_t)d * nq * e, hipMemcpyDeviceToDevice));
        CS_HIP(hipMemcpy(L.wd, s.wd, (size_t)d * F * e, hipMemcpyDeviceToDevice));
        if (c.dtype == CS_BF16)
            k_pack_gu<bf16_t><<<2 * F, 256>>>((const bf16_t*)s.wg, (const bf16_t*)s.wu, F, d,
                                             (bf16_t*)L.wgu);
        else
            k_pack_gu<float><<<2 * F, 256>>>((const float*)s.wg, (const float*)s.wu, F, d,
                                            (float*)L.wgu);
        CS_TRY(cs_launch_ok("k_pack_gu"));
    }
    CS_TRY(weight_range_check(m));          // also waits: the caller's buffers are free again
    if (!m->layer_loaded[l]) { m->layer_loaded[l] = 1; m->layers_loaded += 1; }
    return CS_OK;
}

// storage for the weights and the workspace; the weights come afterwards
static int model_alloc(cs_model* m) {
    const cs_model_cfg& c = m->cfg;
    const size_t e = m->esz;
    const int d = c.d_model, hd = c.head_dim, H = c.n_heads, KVH = c.n_kv_heads, F = c.d_ff,
              V = c.vocab;
    const int nq = H * hd, nkv = KVH * hd, nqkv = nq + 2 * nkv;
    DEV_ALLOC(m->embed, (size_t)V * d * e);
    DEV_ALLOC(m->lm_head, (size_t)V * d * e);
    DEV_ALLOC(m->final_norm, (size_t)d * 4);
    DEV_ALLOC(m->range_flags, 4);
    CS_HIP(hipMemset(m->range_flags, 0, 4));
    for (int l = 0; l < c.n_layers; ++l) {
        cs_layer_dev& L = m->layers[l];
        DEV_ALLOC(L.wqkv, (size_t)nqkv * d * e);
        DEV_ALLOC(L.wo, (size_t)d * nq * e);
        DEV_ALLOC(L.wgu, (size_t)2 * F * d * e);
        DEV_ALLOC(L.wd, (size_t)d * F * e);
        DEV_ALLOC(L.norm1, (size_t)d * 4);
        DEV_ALLOC(L.norm2, (size_t)d * 4);
    }
    // verify blocks have up to R_max rows; prompt blocks of a single stream up to prefill_rows
    const size_t R = (size_t)(m->R_max > m->prefill_rows ? m->R_max : m->prefill_rows);
    const size_t a = m->asz;
    const int wide = d > nq ? d : nq;
    DEV_ALLOC(m->x, R * d * 4);
    DEV_ALLOC(m->xn, R * wide * 4 > cs_xt_bytes(R, wide) ? R * wide * 4 : cs_xt_bytes(R, wide));
    DEV_ALLOC(m->q, R * nq * 4);
    if (!m->fast) DEV_ALLOC(m->gu, R * 2 * F * 4);
    DEV_ALLOC(m->act, R * F * (a > 0 ? a : 4) > cs_xt_bytes(R, F) ? R * F * (a > 0 ? a : 4) : cs_xt_bytes(R, F));
    DEV_ALLOC(m->logits, (size_t)m->R_max * V * 4);
    const int widest = nqkv > d ? nqkv : d;
    m->part_floats = (size_t)16 * R * widest;
    DEV_ALLOC(m->part, m->part_floats * 4);
    const size_t groups_verify = (size_t)c.max_batch * KVH * cs_ceil_div((H / KVH) * m->rows_max, 48);
    // prompt blocks: one stream with prefill_rows rows, or all streams in lock step with
    // their share of the workspace rows each (one more query group per stream from rounding)
    const size_t ws_rows = (size_t)(m->R_max > m->prefill_rows ? m->R_max : m->prefill_rows);
    const size_t groups_prompt = (size_t)KVH * (cs_ceil_div((H / KVH) * ws_rows, 48) + c.max_batch);
    const size_t groups_max = groups_verify > groups_prompt ? groups_verify : groups_prompt;
    m->attn_part_floats = (size_t)(4 * (512 + groups_max) + 64) * 48 * (hd + 2);
    if (m->fast) DEV_ALLOC(m->attn_part, m->attn_part_floats * 4);
    DEV_ALLOC(m->rope, R * (hd / 2) * sizeof(float2));
    DEV_ALLOC(m->tok, R * 4);
    m->am_chunks = 64;                                   // column chunks of the stand-alone argmax
    // ... or one pair per 128-column tile when the lm_head reduces its own tiles
    const size_t am_tiles = cs_ceil_div(V, 128) > m->am_chunks ? (size_t)cs_ceil_div(V, 128) : (size_t)m->am_chunks;
    DEV_ALLOC(m->am_val_idx, (size_t)m->R_max * am_tiles * 2 * 4);
    DEV_ALLOC(m->row_argmax, (size_t)m->R_max * 4);
    DEV_ALLOC(m->draft, (size_t)c.max_batch * (c.max_k > 0 ? c.max_k : 1) * 4);
    DEV_ALLOC(m->draft_len, (size_t)c.max_batch * 4);
    DEV_ALLOC(m->match_pos, (size_t)c.max_batch * 4);
    DEV_ALLOC(m->pending, (size_t)c.max_batch * 4);
    CS_HIP(hipDeviceSynchronize());
    return CS_OK;
}

extern "C" int cs_model_create_staged(const cs_model_cfg* cfg, cs_model** out) {
    CS_REQUIRE(cfg && out, CS_E_ARG, "cs_model_create: NULL argument");
    const cs_model_cfg& c = *cfg;
    CS_REQUIRE(c.n_layers >= 1 && c.d_model >= 1 && c.n_heads >= 1 && c.n_kv_heads >= 1 &&
                   c.head_dim >= 2 && c.d_ff >= 1 && c.vocab >= 1,
               CS_E_ARG, "cs_model_create: non-positive dimension");
    CS_REQUIRE(c.dtype == CS_F32 || c.dtype == CS_BF16, CS_E_ARG, "cs_model_create: bad dtype");
    CS_REQUIRE(c.n_heads % c.n_kv_heads == 0, CS_E_ARG, "n_heads must be a multiple of n_kv_heads");
    CS_REQUIRE(c.head_dim % 2 == 0 && c.head_dim <= 256 && 256 % c.head_dim == 0, CS_E_UNSUPPORTED,
               "head_dim must be a power of two in 2..256");
    CS_REQUIRE(c.d_ff % 16 == 0, CS_E_UNSUPPORTED, "d_ff must be a multiple of 16");
    CS_REQUIRE(c.d_model <= 8192 && c.d_model % 4 == 0, CS_E_UNSUPPORTED,
               "d_model must be a multiple of 4 and <= 8192");
    CS_REQUIRE(c.max_batch >= 1 && c.max_k >= 0 && c.max_k <= 256, CS_E_ARG,
               "max_batch >= 1 and 0 <= max_k <= 256 required");
    cs_model* m = (cs_model*)calloc(1, sizeof(cs_model));
    CS_REQUIRE(m, CS_E_DEVICE, "out of host memory");
    m->cfg = c;
    m->plain = g_plain;
    m->rows_max = c.max_k + 1;
    m->R_max = c.max_batch * m->rows_max;
    const int prompt_rows = g_prompt_rows > 0 ? g_prompt_rows : CS_PROMPT_BLOCK_ROWS;
    m->prefill_rows = m->rows_max > prompt_rows ? m->rows_max : prompt_rows;
    m->esz = c.dtype == CS_BF16 ? 2 : 4;
    const int nq = c.n_heads * c.head_dim;
    m->fast = !m->plain && c.dtype == CS_BF16 && (c.head_dim == 64 || c.head_dim == 128) &&
              c.d_model % 128 == 0 && c.d_ff % 128 == 0 && nq % 128 == 0 && c.vocab % 16 == 0;
    m->asz = m->fast ? 2 : 4;
    m->layers = (cs_layer_dev*)calloc(c.n_layers, sizeof(cs_layer_dev));
    m->layer_loaded = (unsigned char*)calloc(c.n_layers, 1);
    if (!m->layers || !m->layer_loaded) { model_free(m); cs_set_error("out of host memory"); return CS_E_DEVICE; }
    const int rc = model_alloc(m);
    if (rc != CS_OK) { model_free(m); return rc; }
    *out = m;
    return CS_OK;
}

extern "C" int cs_model_load_head(cs_model* m, const void* embed, const void* lm_head, const float* final_norm) {
    CS_REQUIRE(m, CS_E_ARG, "cs_model_load_head: NULL model");
    return model_load_head(m, embed, lm_head, final_norm);
}

extern "C" int cs_model_load_layer(cs_model* m, int32_t layer, const cs_layer_weights* w) {
    CS_REQUIRE(m && w, CS_E_ARG, "cs_model_load_layer: NULL argument");
    CS_REQUIRE(layer >= 0 && layer < m->cfg.n_layers, CS_E_ARG, "layer %d outside 0..%d", layer, m->cfg.n_layers - 1);
    return model_load_layer(m, layer, *w);
}

extern "C" int cs_model_create(const cs_model_cfg* cfg, const cs_weights* w, cs_model** out) {
    CS_REQUIRE(cfg && w && out, CS_E_ARG, "cs_model_create: NULL argument");
    CS_REQUIRE(w->embed && w->lm_head && w->final_norm && w->layers, CS_E_ARG,
               "cs_model_create: NULL weight pointer");
    cs_model* m = nullptr;
    CS_TRY(cs_model_create_staged(cfg, &m));
    int rc = model_load_head(m, w->embed, w->lm_head, w->final_norm);
    for (int l = 0; l < cfg->n_layers && rc == CS_OK; ++l) rc = model_load_layer(m, l, w->layers[l]);
    if (rc != CS_OK) { model_free(m); return rc; }
    *out = m;
    return CS_OK;
}

extern "C" void cs_model_destroy(cs_model* m) {
    if (m) (void)hipDeviceSynchronize();
    model_free(m);
}

extern "C" int cs_model_set_rope_inv_freq(cs_model* m, const double* inv_freq) {
    CS_REQUIRE(m, CS_E_ARG, "cs_model_set_rope_inv_freq: NULL model");
    const int half = m->cfg.head_dim / 2;
    if (inv_freq)
        for (int j = 0; j < half; ++j)
            CS_REQUIRE(std::isfinite(inv_freq[j]), CS_E_ARG, "rotary frequency %d is not finite", j);
    CS_HIP(hipDeviceSynchronize());
    if (!inv_freq) {
        if (m->rope_inv_freq) (void)hipFree(m->rope_inv_freq);
        m->rope_inv_freq = nullptr;
        return CS_OK;
    }
    if (!m->rope_inv_freq) DEV_ALLOC(m->rope_inv_freq, (size_t)half * sizeof(double));
    CS_HIP(hipMemcpy(m->rope_inv_freq, inv_freq, (size_t)half * sizeof(double), hipMemcpyHostToDevice));
    return CS_OK;
}

extern "C" int cs_model_range_status(cs_model* m, int32_t* flags, int32_t clear) {
    CS_REQUIRE(m && flags, CS_E_ARG, "cs_model_range_status: NULL argument");
    CS_HIP(hipDeviceSynchronize());
    CS_HIP(hipMemcpy(flags, m->range_flags, 4, hipMemcpyDeviceToHost));
    if (clear) CS_HIP(hipMemset(m->range_flags, 0, 4));
    return CS_OK;
}

static int range_clear(cs_model* m) {
    CS_HIP(hipDeviceSynchronize());
    CS_HIP(hipMemset(m->range_flags, 0, 4));
    return CS_OK;
}

// the synchronous loops end with this: the tokens are delivered, the status says if they are exact
static int range_check_after_loop(cs_model* m, const char* who) {
    if (!m->fast) return CS_OK;
    int32_t flags = 0;
    CS_TRY(cs_model_range_status(m, &flags, 1));
    CS_REQUIRE(flags == 0, CS_E_RANGE,
               "%s: activations exceeded the float16 range of the projections and were saturated at +-65504 "
               "(flags 0x%x: 1 = RMSNorm output, 2 = attention output, 4 = SwiGLU output); the tokens were "
               "computed from the saturated values", who, flags);
    return CS_OK;
}

// -------------------------------------------------------------------------------------
// KV cache
// -------------------------------------------------------------------------------------
extern "C" int cs_kv_create(const cs_model* m, int32_t batch, int64_t capacity, cs_kv** out) {
    CS_REQUIRE(m && out, CS_E_ARG, "cs_kv_create: NULL argument");
    CS_REQUIRE(batch >= 1 && batch <= m->cfg.max_batch, CS_E_ARG,
               "cs_kv_create: batch %d outside 1..max_batch=%d", batch, m->cfg.max_batch);
    CS_REQUIRE(capacity >= 1 && capacity < (int64_t)1 << 30, CS_E_ARG, "cs_kv_create: bad capacity");
    cs_kv* kv = (cs_kv*)calloc(1, sizeof(cs_kv));
    CS_REQUIRE(kv, CS_E_DEVICE, "out of host memory");
    kv->m = m;
    kv->B = batch;
    kv->limit = cs_round_up(capacity, 64);          // what the capacity checks go by
    kv->cap = cs_round_up(capacity, CS_VBLK);       // what is allocated (the V cache is laid out in blocks)
    const cs_model_cfg& c = m->cfg;
    const size_t bytes = (size_t)c.n_layers * batch * c.n_kv_heads * kv->cap * c.head_dim * m->esz;
    kv->h_len_ub = (int64_t*)calloc(batch, sizeof(int64_t));
    int rc = CS_OK;
    if (!kv->h_len_ub) { cs_set_error("out of host memory"); rc = CS_E_DEVICE; }
    if (rc == CS_OK) rc = dev_alloc(&kv->k, bytes);
    if (rc == CS_OK) rc = dev_alloc(&kv->v, bytes);
    if (rc == CS_OK) rc = dev_alloc((void**)&kv->d_len, (size_t)batch * 4);
    // a history is one token longer than its cache, so the scan of cs_step sees at most limit+1 tokens
    kv->scan_slots = cs_scan_slots(kv->limit + 1);
    if (rc == CS_OK) rc = dev_alloc((void**)&kv->scan_keys, (size_t)batch * kv->scan_slots * sizeof(int64_t));
    // dead rows must hold finite numbers (they are multiplied by zero probabilities)
    if (rc == CS_OK && hipMemset(kv->k, 0, bytes) != hipSuccess) rc = CS_E_DEVICE;
    if (rc == CS_OK && hipMemset(kv->v, 0, bytes) != hipSuccess) rc = CS_E_DEVICE;
    if (rc == CS_OK && hipMemset(kv->d_len, 0, (size_t)batch * 4) != hipSuccess) rc = CS_E_DEVICE;
    if (rc == CS_OK && hipDeviceSynchronize() != hipSuccess) rc = CS_E_DEVICE;
    if (rc != CS_OK) {
        if (g_err[0] == 0) cs_set_error("cs_kv_create: device allocation failed");
        cs_kv_destroy(kv);
        return rc;
    }
    *out = kv;
    return CS_OK;
}

extern "C" void cs_kv_destroy(cs_kv* kv) {
    if (!kv) return;
    (void)hipDeviceSynchronize();
    if (kv->k) (void)hipFree(kv->k);
    if (kv->v) (void)hipFree(kv->v);
    if (kv->d_len) (void)hipFree(kv->d_len);
    if (kv->scan_keys) (void)hipFree(kv->scan_keys);
    free(kv->h_len_ub);
    free(kv);
}

extern "C" int cs_kv_set_len(cs_kv* kv, int32_t b, int64_t len) {
    CS_REQUIRE(kv, CS_E_ARG, "cs_kv_set_len: NULL handle");
    CS_REQUIRE(b >= 0 && b < kv->B, CS_E_ARG, "cs_kv_set_len: stream %d out of range", b);
    CS_REQUIRE(len >= 0 && len <= kv->limit, CS_E_CAPACITY, "cs_kv_set_len: length %lld > capacity",
               (long long)len);
    const int32_t v = (int32_t)len;
    CS_HIP(hipDeviceSynchronize());
    CS_HIP(hipMemcpy(kv->d_len + b, &v, 4, hipMemcpyHostToDevice));
    kv->h_len_ub[b] = len;
    return CS_OK;
}

extern "C" int cs_kv_set_len_dev(cs_kv* kv, const int32_t* d_len, int64_t ub, void* stream) {
    CS_REQUIRE(kv && d_len, CS_E_ARG, "cs_kv_set_len_dev: NULL argument");
    CS_REQUIRE(ub >= 0 && ub <= kv->limit, CS_E_CAPACITY, "cs_kv_set_len_dev: bound %lld > capacity",
               (long long)ub);
    CS_HIP(hipMemcpyAsync(kv->d_len, d_len, (size_t)kv->B * 4, hipMemcpyDeviceToDevice,
                          (hipStream_t)stream));
    for (int b = 0; b < kv->B; ++b) kv->h_len_ub[b] = ub;
    return CS_OK;
}

static int kv_sync_lengths(cs_kv* kv) {
    std::vector<int32_t> h(kv->B);
    CS_HIP(hipDeviceSynchronize());
    CS_HIP(hipMemcpy(h.data(), kv->d_len, (size_t)kv->B * 4, hipMemcpyDeviceToHost));
    for (int b = 0; b < kv->B; ++b) kv->h_len_ub[b] = h[b];
    return CS_OK;
}

extern "C" int64_t cs_kv_len(cs_kv* kv, int32_t b) {
    CS_REQUIRE(kv, CS_E_ARG, "cs_kv_len: NULL handle");
    CS_REQUIRE(b >= 0 && b < kv->B, CS_E_ARG, "cs_kv_len: stream %d out of range", b);
    CS_TRY(kv_sync_lengths(kv));
    return kv->h_len_ub[b];
}

static int kv_io(cs_kv* kv, int layer, int b, int64_t pos0, int64_t n, void* k_rows, void* v_rows,
                 bool to_cache) {
    CS_REQUIRE(kv && k_rows && v_rows, CS_E_ARG, "cs_kv_load/read: NULL argument");
    const cs_model_cfg& c = kv->m->cfg;
    CS_REQUIRE(layer >= 0 && layer < c.n_layers && b >= 0 && b < kv->B, CS_E_ARG,
               "cs_kv_load/read: layer or stream out of range");
    CS_REQUIRE(pos0 >= 0 && n >= 0 && pos0 + n <= kv->limit, CS_E_CAPACITY,
               "cs_kv_load/read: rows [%lld, %lld) exceed capacity %lld", (long long)pos0,
               (long long)(pos0 + n), (long long)kv->limit);
    if (n == 0) return CS_OK;
    const size_t e = kv->m->esz;
    const int hd = c.head_dim, KVH = c.n_kv_heads;
    const int64_t item = ((int64_t)layer * kv->B + b) * KVH;
    char* kc = (char*)kv->k + (item * kv->cap + pos0) * hd * e;
    if (to_cache)
        CS_HIP(hipMemcpy2D(kc, (size_t)kv->cap * hd * e, k_rows, (size_t)n * hd * e, (size_t)n * hd * e,
                           KVH, hipMemcpyDeviceToDevice));
    else
        CS_HIP(hipMemcpy2D(k_rows, (size_t)n * hd * e, kc, (size_t)kv->cap * hd * e, (size_t)n * hd * e,
                           KVH, hipMemcpyDeviceToDevice));
    char* vc = (char*)kv->v + item * hd * kv->cap * e;
    dim3 grid((unsigned)(cs_ceil_div(n * hd, 256) < 1024 ? cs_ceil_div(n * hd, 256) : 1024), KVH);
    if (c.dtype == CS_BF16) {
        if (to_cache) k_v_transpose<bf16_t, 1><<<grid, 256>>>((bf16_t*)vc, (bf16_t*)v_rows, kv->cap, hd, pos0, n);
        else k_v_transpose<bf16_t, 0><<<grid, 256>>>((bf16_t*)vc, (bf16_t*)v_rows, kv->cap, hd, pos0, n);
    } else {
        if (to_cache) k_v_transpose<float, 1><<<grid, 256>>>((float*)vc, (float*)v_rows, kv->cap, hd, pos0, n);
        else k_v_transpose<float, 0><<<grid, 256>>>((float*)vc, (float*)v_rows, kv->cap, hd, pos0, n);
    }
    CS_TRY(cs_launch_ok("k_v_transpose"));
    CS_HIP(hipDeviceSynchronize());
    return CS_OK;
}

extern "C" int cs_kv_load(cs_kv* kv, int32_t layer, int32_t b, int64_t pos0, int64_t n,
                          const void* k_rows, const void* v_rows) {
    return kv_io(kv, layer, b, pos0, n, (void*)k_rows, (void*)v_rows, true);
}
extern "C" int cs_kv_read(cs_kv* kv, int32_t layer, int32_t b, int64_t pos0, int64_t n, void* k_rows,
                          void* v_rows) {
    return kv_io(kv, layer, b, pos0, n, k_rows, v_rows, false);
}

// -------------------------------------------------------------------------------------
// match search entry points
// -------------------------------------------------------------------------------------
int cs_check_scan_args(int gamma, int k, int policy) {
    CS_REQUIRE(gamma >= 1 && gamma <= 16, CS_E_ARG, "gamma must be in 1..16 (got %d)", gamma);
    CS_REQUIRE(k >= 0 && k <= 256, CS_E_ARG, "k must be in 0..256 (got %d)", k);
    CS_REQUIRE(policy == CS_POLICY_RIGHTMOST || policy == CS_POLICY_FIRST || policy == CS_POLICY_CONTEXT,
               CS_E_ARG, "unknown match policy %d", policy);
    return CS_OK;
}

extern "C" int cs_find_match_batch_dev(const int32_t* d_hist, int64_t stride, const int32_t* d_len,
                                       int32_t B, int32_t gamma, int32_t k, int32_t policy,
                                       int32_t* d_match_pos, int32_t* d_src_pos, int32_t* d_draft,
                                       int32_t* d_draft_len, void* stream) {
    CS_TRY(cs_check_scan_args(gamma, k, policy));
    CS_REQUIRE(B >= 0, CS_E_ARG, "B must be >= 0");
    if (B == 0) return CS_OK;
    CS_REQUIRE(d_hist && d_len && d_draft_len && (d_draft || k == 0), CS_E_ARG,
               "cs_find_match_batch_dev: NULL pointer");
    CS_REQUIRE(stride >= 1 && stride <= CS_MAX_STRIDE, CS_E_ARG, "stride out of range");
    CS_REQUIRE(B <= 65535, CS_E_ARG, "at most 65535 histories per call");
    const int nslots = cs_scan_slots(stride);
    int64_t* keys = nullptr;
    CS_TRY(cs_scan_stream_keys((size_t)B * nslots, (hipStream_t)stream, &keys));
    return cs_scan_launch(d_hist, stride, d_len, B, gamma, k, policy, keys, nslots, d_match_pos, d_src_pos,
                          d_draft, d_draft_len, nullptr, (hipStream_t)stream);
}

extern "C" int cs_find_match_ex(const int32_t* history, int64_t len, int32_t gamma, int32_t k,
                                int32_t policy, int64_t* match_pos, int64_t* src_pos, int32_t* draft,
                                int32_t* draft_len) {
    CS_TRY(cs_check_scan_args(gamma, k, policy));
    CS_REQUIRE(len >= 0 && len <= CS_MAX_STRIDE, CS_E_ARG, "history length out of range");
    CS_REQUIRE(history || len == 0, CS_E_ARG, "cs_find_match: NULL history");
    int32_t out[3] = {-1, -1, 0};
    std::vector<int32_t> hdraft((size_t)(k > 0 ? k : 1), -1);
    if (len >= 2 * (int64_t)gamma) {
        const int64_t stride = cs_round_up(len, 4);
        int32_t* d = nullptr;
        // history | len, match, src, draft_len | draft | per-chunk keys (8-byte aligned)
        const int nslots = cs_scan_slots(len);
        const size_t words = (size_t)cs_round_up(stride + 4 + (k > 0 ? k : 1), 2);
        CS_HIP(hipMalloc(&d, words * 4 + (size_t)nslots * sizeof(int64_t)));
        int32_t* d_len = d + stride;
        int32_t* d_out = d_len + 1;         // match, src, draft_len
        int32_t* d_draft = d_out + 3;
        int64_t* d_keys = reinterpret_cast<int64_t*>(d + words);
        const int32_t n32 = (int32_t)len;
        int rc = CS_OK;
        if (hipMemcpy(d, history, (size_t)len * 4, hipMemcpyHostToDevice) != hipSuccess ||
            hipMemcpy(d_len, &n32, 4, hipMemcpyHostToDevice) != hipSuccess) {
            cs_set_error("cs_find_match: copy to device failed");
            rc = CS_E_DEVICE;
        }
        if (rc == CS_OK)
            rc = cs_scan_launch(d, stride, d_len, 1, gamma, k, policy, d_keys, nslots, d_out, d_out + 1,
                                d_draft, d_out + 2, nullptr, nullptr);
        if (rc == CS_OK && (hipMemcpy(out, d_out, 12, hipMemcpyDeviceToHost) != hipSuccess ||
                            (k > 0 && hipMemcpy(hdraft.data(), d_draft, (size_t)k * 4,
                                                hipMemcpyDeviceToHost) != hipSuccess))) {
            cs_set_error("cs_find_match: copy from device failed");
            rc = CS_E_DEVICE;
        }
        (void)hipFree(d);
        if (rc != CS_OK) return rc;
    }
    if (match_pos) *match_pos = out[0];
    if (src_pos) *src_pos = out[1];
    if (draft_len) *draft_len = out[2];
    if (draft)
        for (int i = 0; i < k; ++i) draft[i] = hdraft[i];
    return CS_OK;
}

extern "C" int64_t cs_find_match(const int32_t* history, int64_t len, int32_t gamma) {
    int64_t src = -1;
    const int rc = cs_find_match_ex(history, len, gamma, 0, CS_POLICY_RIGHTMOST, nullptr, &src,
                                    nullptr, nullptr);
    return rc == CS_OK ? src : (int64_t)rc;
}

// -------------------------------------------------------------------------------------
// verify pass
// -------------------------------------------------------------------------------------
static int64_t kv_max_ub(const cs_kv* kv) {
    int64_t mx = 0;
    for (int b = 0; b < kv->B; ++b) mx = kv->h_len_ub[b] > mx ? kv->h_len_ub[b] : mx;
    return mx;
}

// key slots per stream for a scan of this cache's histories (one token longer than the cache rows)
static int kv_scan_slots(const cs_kv* kv) {
    const int want = cs_scan_slots(kv_max_ub(kv) + 1);
    return want < kv->scan_slots ? want : kv->scan_slots;
}

// every stream must have room for `rows` more rows; refreshes the host bounds if needed
static int kv_check_room(cs_kv* kv, int rows) {
    if (kv_max_ub(kv) + rows > kv->limit) CS_TRY(kv_sync_lengths(kv));
    CS_REQUIRE(kv_max_ub(kv) + rows <= kv->limit, CS_E_CAPACITY,
               "KV cache full: length %lld + %d rows > capacity %lld", (long long)kv_max_ub(kv), rows,
               (long long)kv->limit);
    return CS_OK;
}

// m->tok holds the block tokens; runs all layers; leaves the final-normed rows in m->xn
static int forward_layers(cs_model* m, cs_kv* kv, int rows, hipStream_t s) {
    const cs_model_cfg& c = m->cfg;
    const int B = kv->B, R = B * rows;
    const int d = c.d_model, nq = c.n_heads * c.head_dim, nqkv = nq + 2 * c.n_kv_heads * c.head_dim;
    const int64_t len_ub = kv_max_ub(kv);
    CS_REQUIRE(m->head_loaded && m->layers_loaded == c.n_layers, CS_E_STATE,
               "the model is not complete: %d of %d layers loaded, embedding and lm_head %s", m->layers_loaded,
               c.n_layers, m->head_loaded ? "loaded" : "missing");
    CS_TRY(cs_rope_table_launch(m, kv->d_len, B, rows, s));
    CS_TRY(cs_embed_launch(m, m->tok, R, s));
    int np_prev = 0, np = 1;
    // narrow blocks: the attention kernel rotates q and k and appends k, v itself
    const bool fuse_rope = cs_attention_fuses_rope(m, rows);
    for (int l = 0; l < c.n_layers; ++l) {
        const cs_layer_dev& L = m->layers[l];
        CS_TRY(cs_addnorm_launch(m, m->part, np_prev, L.norm1, m->xn, R, nqkv, s));
        CS_TRY(cs_gemm_launch(m, m->xn, L.wqkv, m->part, R, nqkv, d, CS_GEMM_STORE, 1, &np, s));
        if (fuse_rope) {
            CS_TRY(cs_attention_launch(m, kv, l, rows, len_ub, 1, m->part, np, s));
        } else {
            CS_TRY(cs_rope_append_launch(m, kv, l, m->part, np, rows, s));
            CS_TRY(cs_attention_launch(m, kv, l, rows, len_ub, 1, nullptr, 0, s));
        }
        CS_TRY(cs_gemm_launch(m, m->xn, L.wo, m->part, R, d, nq, CS_GEMM_STORE, 1, &np, s));
        CS_TRY(cs_addnorm_launch(m, m->part, np, L.norm2, m->xn, R, 2 * c.d_ff, s));
        if (m->fast) {
            CS_TRY(cs_gemm_launch(m, m->xn, L.wgu, nullptr, R, 2 * c.d_ff, d, CS_GEMM_SWIGLU, 0,
                                  nullptr, s));
        } else {
            CS_TRY(cs_gemm_launch(m, m->xn, L.wgu, m->gu, R, 2 * c.d_ff, d, CS_GEMM_STORE, 0, nullptr, s));
            CS_TRY(cs_swiglu_launch(m, R, s));
        }
        CS_TRY(cs_gemm_launch(m, m->act, L.wd, m->part, R, d, c.d_ff, CS_GEMM_STORE, 1, &np_prev, s));
    }
    // the final norm feeds the lm_head (callers that only fill the cache never read it)
    return cs_addnorm_launch(m, m->part, np_prev, m->final_norm, m->xn, R, c.vocab, s);
}

static int verify_impl(cs_model* m, cs_kv* kv, const int32_t* d_pending, const int32_t* d_draft,
                       const int32_t* d_draft_len, int k, int32_t* d_accepted, int32_t* d_next,
                       float* d_logits_out, int32_t* hist, int64_t hist_stride, int32_t* hist_len,
                       int32_t* room, hipStream_t s) {
    const int rows = k + 1, B = kv->B, R = B * rows, V = m->cfg.vocab;
    CS_TRY(kv_check_room(kv, rows));
    CS_TRY(cs_tokens_launch(m, d_pending, d_draft, d_draft_len, B, k, s));
    CS_TRY(forward_layers(m, kv, rows, s));
    const int pl = cs_prof_begin(CS_PROF_LMHEAD, s);
    if (m->fast && !d_logits_out) {
        // nobody wants the logits: the lm_head keeps them in its accumulators and hands over the
        // largest entry of every row per column tile; the accept kernel finishes the argmax
        int nch = 0;
        CS_TRY(cs_gemm_launch(m, m->xn, m->lm_head, nullptr, R, V, m->cfg.d_model, CS_GEMM_ARGMAX, 0,
                              &nch, s));
        cs_prof_end(pl, s);
        CS_TRY(cs_accept_launch(m, nch, B, k, d_draft, d_draft_len, d_accepted, d_next, nullptr,
                                kv->d_len, hist, hist_stride, hist_len, room, s));
    } else {
        CS_TRY(cs_gemm_launch(m, m->xn, m->lm_head, m->logits, R, V, m->cfg.d_model, CS_GEMM_STORE, 0,
                              nullptr, s));
        cs_prof_end(pl, s);
        CS_TRY(cs_argmax_accept_launch(m, m->logits, B, k, V, d_draft, d_draft_len, d_accepted, d_next,
                                       nullptr, kv->d_len, hist, hist_stride, hist_len, room, s));
    }
    if (d_logits_out)
        CS_HIP(hipMemcpyAsync(d_logits_out, m->logits, (size_t)R * V * 4, hipMemcpyDeviceToDevice, s));
    for (int b = 0; b < B; ++b) kv->h_len_ub[b] += rows;
    return CS_OK;
}

static int check_verify_args(cs_model* m, cs_kv* kv, int k) {
    CS_REQUIRE(m && kv, CS_E_ARG, "NULL model or kv handle");
    CS_REQUIRE(kv->m == m, CS_E_STATE, "kv cache belongs to a different model");
    CS_REQUIRE(k >= 0 && k <= m->cfg.max_k, CS_E_ARG, "k=%d outside 0..max_k=%d", k, m->cfg.max_k);
    return CS_OK;
}

extern "C" int cs_verify(cs_model* m, cs_kv* kv, const int32_t* d_pending, const int32_t* d_draft,
                         const int32_t* d_draft_len, int32_t k, int32_t* d_accepted_len,
                         int32_t* d_next_token, float* d_logits_out, void* stream) {
    CS_TRY(check_verify_args(m, kv, k));
    CS_REQUIRE(d_pending && d_draft_len && d_accepted_len && d_next_token && (d_draft || k == 0),
               CS_E_ARG, "cs_verify: NULL pointer");
    return verify_impl(m, kv, d_pending, d_draft, d_draft_len, k, d_accepted_len, d_next_token,
                       d_logits_out, nullptr, 0, nullptr, nullptr, (hipStream_t)stream);
}

extern "C" int cs_step(cs_model* m, cs_kv* kv, int32_t* d_hist, int64_t stride, int32_t* d_hist_len,
                       int32_t* d_room, int32_t gamma, int32_t k, int32_t policy,
                       int32_t* d_accepted_len, int32_t* d_next_token, int32_t* d_draft_len_out,
                       void* stream) {
    CS_TRY(check_verify_args(m, kv, k));
    CS_TRY(cs_check_scan_args(gamma, k, policy));
    CS_REQUIRE(d_hist && d_hist_len && d_accepted_len && d_next_token, CS_E_ARG, "cs_step: NULL pointer");
    CS_REQUIRE(stride >= 1 && stride <= CS_MAX_STRIDE, CS_E_ARG, "stride out of range");
    hipStream_t s = (hipStream_t)stream;
    const int B = kv->B;
    CS_TRY(kv_check_room(kv, k + 1));
    // the history may grow by k+1 tokens: same bound as the cache (length = kv length + 1)
    CS_REQUIRE(kv_max_ub(kv) + 1 + k + 1 <= stride, CS_E_CAPACITY,
               "history buffer (stride %lld) may overflow", (long long)stride);
    if (k > 0) {
        CS_TRY(cs_scan_launch(d_hist, stride, d_hist_len, B, gamma, k, policy, kv->scan_keys,
                              kv_scan_slots(kv), m->match_pos, nullptr, m->draft, m->draft_len, d_room, s));
    } else {
        CS_TRY(cs_fill_i32_launch(m->draft_len, 0, B, s));
    }
    k_pending<<<(unsigned)cs_ceil_div(B, 64), 64, 0, s>>>(d_hist, stride, d_hist_len, B, m->pending);
    CS_TRY(cs_launch_ok("k_pending"));
    if (d_draft_len_out)
        CS_HIP(hipMemcpyAsync(d_draft_len_out, m->draft_len, (size_t)B * 4, hipMemcpyDeviceToDevice, s));
    return verify_impl(m, kv, m->pending, m->draft, m->draft_len, k, d_accepted_len, d_next_token,
                       nullptr, d_hist, stride, d_hist_len, d_room, s);
}

// -------------------------------------------------------------------------------------
// prefill and decode loops
// -------------------------------------------------------------------------------------
extern "C" int cs_prefill(cs_model* m, cs_kv* kv, int32_t stream_idx, const int32_t* prompt,
                          int64_t prompt_len) {
    CS_REQUIRE(m && kv && prompt, CS_E_ARG, "cs_prefill: NULL argument");
    CS_REQUIRE(kv->m == m, CS_E_STATE, "kv cache belongs to a different model");
    CS_REQUIRE(kv->B == 1 && stream_idx == 0, CS_E_UNSUPPORTED,
               "cs_prefill supports single-stream caches only");
    CS_REQUIRE(prompt_len >= 1, CS_E_ARG, "prompt must hold at least one token");
    CS_REQUIRE(prompt_len - 1 <= kv->limit, CS_E_CAPACITY, "prompt longer than the cache");
    for (int64_t i = 0; i < prompt_len; ++i)
        CS_REQUIRE(prompt[i] >= 0 && prompt[i] < m->cfg.vocab, CS_E_ARG,
                   "prompt token %lld out of vocabulary", (long long)i);
    CS_TRY(cs_kv_set_len(kv, 0, 0));
    const int64_t body = prompt_len - 1;
    const int chunk = m->prefill_rows;
    for (int64_t c0 = 0; c0 < body; c0 += chunk) {
        const int rows = (int)(body - c0 < chunk ? body - c0 : chunk);
        CS_HIP(hipMemcpyAsync(m->tok, prompt + c0, (size_t)rows * 4, hipMemcpyHostToDevice, nullptr));
        CS_TRY(forward_layers(m, kv, rows, nullptr));
        k_add_i32<<<1, 64, 0, nullptr>>>(kv->d_len, rows, 1);
        CS_TRY(cs_launch_ok("k_add_i32"));
        kv->h_len_ub[0] += rows;
    }
    CS_HIP(hipDeviceSynchronize());
    return CS_OK;
}

// Steps the decode loops enqueue between two host reads.  A step whose streams have used up
// their budgets still costs a forward pass, so a burst never holds more steps than the stream
// with the most tokens left needs at full acceptance; only a stop token can make the tail of
// a burst idle.
static const int DECODE_BURST = 4;

// room for the histories of a decode loop: every step of a burst is checked against the host's
// upper bound of the lengths, which grows by k+1 per step until the next read
static int64_t decode_stride(int64_t max_len, int64_t max_new, int k) {
    return cs_round_up(max_len + max_new + (int64_t)DECODE_BURST * (k + 1) + 2, 4);
}

// The loop of cs_decode and cs_decode_batch (Sec. 3.2; App. B.3 step 4): cs_step on all streams
// of a prefilled cache until every stream has emitted max_new tokens or eos_id.  d_hist holds
// the prompts ([B][stride], device); lengths, budgets and the outcome of every step stay on
// the device, and the host reads the log of a whole burst of steps in one copy.
static int decode_loop(cs_model* m, cs_kv* kv, int32_t* d_hist, int64_t stride,
                       const int64_t* prompt_len, int64_t max_new, int gamma, int k, int policy,
                       int eos_id, int32_t* out_tokens, int64_t* emitted, cs_stats* st) {
    const int B = kv->B;
    // device state: [hist_len | room] (B each), then per step of a burst
    // [accepted | next | draft_len] (B each) and the tokens the step appended [B][k+1]
    const size_t n_slice = (size_t)3 * B + (size_t)B * (k + 1);
    const size_t n_state = (size_t)2 * B + (size_t)DECODE_BURST * n_slice;
    int32_t* d_state = nullptr;
    CS_HIP(hipMalloc(&d_state, n_state * 4));
    std::vector<int32_t> h(n_state, 0);
    std::vector<char> active((size_t)B, max_new > 0 ? 1 : 0);
    for (int b = 0; b < B; ++b) {
        h[b] = (int32_t)prompt_len[b];
        h[B + b] = (int32_t)max_new;
        emitted[b] = 0;
        st[b] = cs_stats{0, 0, 0, 0};
    }
    int rc = CS_OK;
    if (hipMemcpy(d_state, h.data(), (size_t)2 * B * 4, hipMemcpyHostToDevice) != hipSuccess) {
        cs_set_error("decode loop: copy to device failed");
        rc = CS_E_DEVICE;
    }
    while (rc == CS_OK) {
        int64_t most = 0;
        for (int b = 0; b < B; ++b)
            if (active[b] && max_new - emitted[b] > most) most = max_new - emitted[b];
        if (most == 0) break;
        const int64_t need = cs_ceil_div(most, (int64_t)k + 1);
        const int burst = (int)(need < DECODE_BURST ? need : DECODE_BURST);
        for (int j = 0; j < burst && rc == CS_OK; ++j) {
            int32_t* sl = d_state + 2 * B + (size_t)j * n_slice;
            rc = cs_step(m, kv, d_hist, stride, d_state, d_state + B, gamma, k, policy, sl, sl + B,
                         sl + 2 * B, nullptr);
            if (rc != CS_OK) break;
            k_emitted<<<B, 64, 0, nullptr>>>(d_hist, stride, d_state, sl, k, sl + 3 * B);
            rc = cs_launch_ok("k_emitted");
        }
        if (rc != CS_OK) break;
        if (hipMemcpy(h.data(), d_state, ((size_t)2 * B + (size_t)burst * n_slice) * 4,
                      hipMemcpyDeviceToHost) != hipSuccess) {
            cs_set_error("decode loop: copy from device failed");
            rc = CS_E_DEVICE;
            break;
        }
        for (int b = 0; b < B; ++b) kv->h_len_ub[b] = h[b] - 1;   // everything but the pending token
        for (int j = 0; j < burst; ++j) {
            const int32_t* sl = h.data() + 2 * B + (size_t)j * n_slice;
            for (int b = 0; b < B; ++b) {
                if (!active[b]) continue;
                const int tau = sl[b], got = tau + 1, dl = sl[2 * B + b];
                const int32_t* fresh = sl + 3 * B + (size_t)b * (k + 1);
                st[b].steps += 1;
                if (dl > 0) { st[b].attempts += 1; st[b].drafted += dl; st[b].accepted += tau; }
                int take = got;
                bool stopped = false;
                for (int i = 0; i < got; ++i)
                    if (eos_id >= 0 && fresh[i] == eos_id) { take = i + 1; stopped = true; break; }
                for (int i = 0; i < take; ++i) out_tokens[(int64_t)b * max_new + emitted[b] + i] = fresh[i];
                emitted[b] += take;
                if (stopped || emitted[b] >= max_new) active[b] = 0;
                if (stopped) {
                    // the steps after the stop token are not part of the output: the stream's budget
                    // goes to 0 and its cache back to the tokens before the stop token
                    const int32_t zero = 0;
                    const int64_t keep = prompt_len[b] + emitted[b] - 1;
                    if (hipMemcpy(d_state + B + b, &zero, 4, hipMemcpyHostToDevice) != hipSuccess) {
                        cs_set_error("decode loop: copy to device failed");
                        rc = CS_E_DEVICE;
                    } else {
                        rc = cs_kv_set_len(kv, b, keep);
                    }
                    if (rc != CS_OK) break;
                }
            }
            if (rc != CS_OK) break;
        }
    }
    (void)hipFree(d_state);
    return rc;
}

static int decode_impl(cs_model* m, cs_kv* kv, const int32_t* prompt, int64_t prompt_len,
                       int64_t max_new, int gamma, int k, int policy, int eos_id, int32_t* out_tokens,
                       int64_t* n_out, cs_stats* stats) {
    CS_REQUIRE(out_tokens && n_out, CS_E_ARG, "cs_decode: NULL output");
    CS_REQUIRE(max_new >= 0, CS_E_ARG, "max_new must be >= 0");
    CS_TRY(check_verify_args(m, kv, k));
    CS_REQUIRE(kv->B == 1, CS_E_UNSUPPORTED, "cs_decode needs a single-stream cache");
    CS_REQUIRE(prompt && prompt_len >= 1, CS_E_ARG, "prompt must hold at least one token");
    CS_REQUIRE(prompt_len + max_new + k + 1 <= kv->limit, CS_E_CAPACITY,
               "cache capacity %lld < prompt_len + max_new + k + 1", (long long)kv->limit);
    *n_out = 0;
    CS_TRY(range_clear(m));
    CS_TRY(cs_prefill(m, kv, 0, prompt, prompt_len));
    const int64_t stride = decode_stride(prompt_len, max_new, k);
    CS_REQUIRE(stride <= CS_MAX_STRIDE, CS_E_ARG, "history too long");
    int32_t* d = nullptr;
    CS_HIP(hipMalloc(&d, (size_t)stride * 4));
    int rc = CS_OK;
    if (hipMemcpy(d, prompt, (size_t)prompt_len * 4, hipMemcpyHostToDevice) != hipSuccess) {
        cs_set_error("cs_decode: copy to device failed");
        rc = CS_E_DEVICE;
    }
    int64_t emitted = 0;
    cs_stats st = {0, 0, 0, 0};
    if (rc == CS_OK)
        rc = decode_loop(m, kv, d, stride, &prompt_len, max_new, gamma, k, policy, eos_id, out_tokens,
                         &emitted, &st);
    (void)hipFree(d);
    if (rc != CS_OK) return rc;
    *n_out = emitted;
    if (stats) *stats = st;
    return range_check_after_loop(m, "cs_decode");
}

extern "C" int cs_decode(cs_model* m, cs_kv* kv, const int32_t* prompt, int64_t prompt_len,
                         int64_t max_new, int32_t gamma, int32_t k, int32_t policy, int32_t eos_id,
                         int32_t* out_tokens, int64_t* n_out, cs_stats* stats) {
    CS_TRY(cs_check_scan_args(gamma, k, policy));
    return decode_impl(m, kv, prompt, prompt_len, max_new, gamma, k, policy, eos_id, out_tokens, n_out,
                       stats);
}

extern "C" int cs_decode_greedy(cs_model* m, cs_kv* kv, const int32_t* prompt, int64_t prompt_len,
                                int64_t max_new, int32_t eos_id, int32_t* out_tokens, int64_t* n_out) {
    return decode_impl(m, kv, prompt, prompt_len, max_new, 1, 0, CS_POLICY_RIGHTMOST, eos_id,
                       out_tokens, n_out, nullptr);
}

// -------------------------------------------------------------------------------------
// all streams of a cache at once
// -------------------------------------------------------------------------------------
static int check_prompts(const cs_model* m, const cs_kv* kv, const int32_t* prompts, int64_t stride,
                         const int64_t* prompt_len, int64_t* max_len_out) {
    CS_REQUIRE(prompts && prompt_len, CS_E_ARG, "NULL prompt argument");
    int64_t max_len = 0;
    for (int b = 0; b < kv->B; ++b) {
        CS_REQUIRE(prompt_len[b] >= 1, CS_E_ARG, "prompt %d must hold at least one token", b);
        CS_REQUIRE(prompt_len[b] <= stride, CS_E_ARG, "prompt %d is longer than prompt_stride", b);
        CS_REQUIRE(prompt_len[b] - 1 <= kv->limit, CS_E_CAPACITY, "prompt %d longer than the cache", b);
        max_len = prompt_len[b] > max_len ? prompt_len[b] : max_len;
        for (int64_t i = 0; i < prompt_len[b]; ++i) {
            const int32_t t = prompts[(int64_t)b * stride + i];
            CS_REQUIRE(t >= 0 && t < m->cfg.vocab, CS_E_ARG, "prompt %d token %lld out of vocabulary", b,
                       (long long)i);
        }
    }
    *max_len_out = max_len;
    return CS_OK;
}

extern "C" int cs_prefill_batch(cs_model* m, cs_kv* kv, const int32_t* prompts, int64_t prompt_stride,
                                const int64_t* prompt_len) {
    CS_REQUIRE(m && kv, CS_E_ARG, "cs_prefill_batch: NULL handle");
    CS_REQUIRE(kv->m == m, CS_E_STATE, "kv cache belongs to a different model");
    int64_t max_len = 0;
    CS_TRY(check_prompts(m, kv, prompts, prompt_stride, prompt_len, &max_len));
    const int B = kv->B;
    CS_HIP(hipDeviceSynchronize());
    CS_HIP(hipMemset(kv->d_len, 0, (size_t)B * 4));
    for (int b = 0; b < B; ++b) kv->h_len_ub[b] = 0;
    // Lock step: every pass runs the same number of rows for every stream.  A stream whose
    // prompt is used up rides along on padding rows; their cache entries land beyond its
    // length (dead rows) and, the block being causal, no live row ever sees them.
    const int64_t ws_rows = m->R_max > m->prefill_rows ? m->R_max : m->prefill_rows;
    const int64_t chunk = ws_rows / B > 0 ? ws_rows / B : 1;
    const int64_t max_body = max_len - 1;
    std::vector<int32_t> tok, inc((size_t)B);
    int32_t* d_inc = nullptr;
    CS_HIP(hipMalloc(&d_inc, (size_t)B * 4));
    int rc = CS_OK;
    for (int64_t c0 = 0; c0 < max_body && rc == CS_OK; c0 += chunk) {
        const int rows = (int)(max_body - c0 < chunk ? max_body - c0 : chunk);
        tok.assign((size_t)B * rows, 0);
        for (int b = 0; b < B; ++b) {
            const int64_t left = prompt_len[b] - 1 - c0;
            const int64_t live = left < 0 ? 0 : (left < rows ? left : rows);
            for (int64_t i = 0; i < live; ++i) tok[(size_t)b * rows + i] = prompts[(int64_t)b * prompt_stride + c0 + i];
            inc[b] = (int32_t)live;
        }
        if (hipMemcpy(m->tok, tok.data(), tok.size() * 4, hipMemcpyHostToDevice) != hipSuccess ||
            hipMemcpy(d_inc, inc.data(), (size_t)B * 4, hipMemcpyHostToDevice) != hipSuccess) {
            cs_set_error("cs_prefill_batch: copy to device failed");
            rc = CS_E_DEVICE;
            break;
        }
        rc = forward_layers(m, kv, rows, nullptr);
        if (rc != CS_OK) break;
        k_add_i32_vec<<<(unsigned)cs_ceil_div(B, 64), 64, 0, nullptr>>>(kv->d_len, d_inc, B);
        rc = cs_launch_ok("k_add_i32_vec");
        for (int b = 0; b < B; ++b) kv->h_len_ub[b] += inc[b];
    }
    if (hipDeviceSynchronize() != hipSuccess && rc == CS_OK) {
        cs_set_error("cs_prefill_batch: device error");
        rc = CS_E_DEVICE;
    }
    (void)hipFree(d_inc);
    return rc;
}

extern "C" int cs_decode_batch(cs_model* m, cs_kv* kv, const int32_t* prompts, int64_t prompt_stride,
                               const int64_t* prompt_len, int64_t max_new, int32_t gamma, int32_t k,
                               int32_t policy, int32_t eos_id, int32_t* out_tokens, int64_t* n_out,
                               cs_stats* stats) {
    CS_REQUIRE(out_tokens && n_out, CS_E_ARG, "cs_decode_batch: NULL output");
    CS_REQUIRE(max_new >= 0, CS_E_ARG, "max_new must be >= 0");
    CS_TRY(cs_check_scan_args(gamma, k, policy));
    CS_TRY(check_verify_args(m, kv, k));
    const int B = kv->B;
    int64_t max_len = 0;
    CS_TRY(check_prompts(m, kv, prompts, prompt_stride, prompt_len, &max_len));
    CS_REQUIRE(max_len + max_new + k + 1 <= kv->limit, CS_E_CAPACITY,
               "cache capacity %lld < longest prompt + max_new + k + 1", (long long)kv->limit);
    std::vector<cs_stats> st((size_t)B, cs_stats{0, 0, 0, 0});
    std::vector<int64_t> emitted((size_t)B, 0);
    for (int b = 0; b < B; ++b) n_out[b] = 0;
    CS_TRY(range_clear(m));
    CS_TRY(cs_prefill_batch(m, kv, prompts, prompt_stride, prompt_len));
    const int64_t stride = decode_stride(max_len, max_new, k);
    CS_REQUIRE(stride <= CS_MAX_STRIDE, CS_E_ARG, "history too long");
    int32_t* d = nullptr;
    CS_HIP(hipMalloc(&d, (size_t)B * stride * 4));
    int rc = CS_OK;
    if (hipMemcpy2D(d, (size_t)stride * 4, prompts, (size_t)prompt_stride * 4, (size_t)max_len * 4, B,
                    hipMemcpyHostToDevice) != hipSuccess) {
        cs_set_error("cs_decode_batch: copy to device failed");
        rc = CS_E_DEVICE;
    }
    if (rc == CS_OK)
        rc = decode_loop(m, kv, d, stride, prompt_len, max_new, gamma, k, policy, eos_id, out_tokens,
                         emitted.data(), st.data());
    (void)hipFree(d);
    if (rc != CS_OK) return rc;
    for (int b = 0; b < B; ++b) {
        n_out[b] = emitted[b];
        if (stats) stats[b] = st[b];
    }
    return range_check_after_loop(m, "cs_decode_batch");
}

// -------------------------------------------------------------------------------------
// CopySpec merged with draft-model speculative decoding (Sec. 3.3, App. B.3 steps 1-4)
// -------------------------------------------------------------------------------------
extern "C" int cs_decode_merged(cs_model* m, cs_kv* kv, cs_model* dm, cs_kv* dkv, const int32_t* prompt,
                                int64_t prompt_len, int64_t max_new, int32_t gamma, int32_t k,
                                int32_t policy, int32_t delta, int32_t eos_id, int32_t* out_tokens,
                                int64_t* n_out, cs_merged_stats* stats) {
    CS_REQUIRE(out_tokens && n_out, CS_E_ARG, "cs_decode_merged: NULL output");
    CS_REQUIRE(max_new >= 0, CS_E_ARG, "max_new must be >= 0");
    CS_TRY(cs_check_scan_args(gamma, k, policy));
    CS_TRY(check_verify_args(m, kv, k));
    CS_REQUIRE(dm && dkv && dkv->m == dm, CS_E_ARG, "cs_decode_merged: draft model and its cache do not match");
    CS_REQUIRE(dm != m && dkv != kv, CS_E_ARG, "the draft model needs a model handle and a cache of its own");
    CS_REQUIRE(dm->cfg.vocab == m->cfg.vocab, CS_E_ARG, "draft and target vocabularies differ (%d vs %d)",
               dm->cfg.vocab, m->cfg.vocab);
    CS_REQUIRE(delta >= 0 && delta <= m->cfg.max_k, CS_E_ARG, "delta=%d outside 0..max_k=%d", delta,
               m->cfg.max_k);
    CS_REQUIRE(kv->B == 1 && dkv->B == 1, CS_E_UNSUPPORTED, "cs_decode_merged needs single-stream caches");
    CS_REQUIRE(prompt && prompt_len >= 1, CS_E_ARG, "prompt must hold at least one token");
    const int kmax = k > delta ? k : delta;
    CS_REQUIRE(prompt_len + max_new + kmax + 1 <= kv->limit, CS_E_CAPACITY,
               "target cache capacity %lld < prompt_len + max_new + max(k, delta) + 1", (long long)kv->limit);
    CS_REQUIRE(prompt_len + max_new + delta + 1 <= dkv->limit, CS_E_CAPACITY,
               "draft cache capacity %lld < prompt_len + max_new + delta + 1", (long long)dkv->limit);
    cs_merged_stats st = {0, 0, 0, 0, 0, 0, 0, 0};
    *n_out = 0;
    CS_TRY(range_clear(m));
    CS_TRY(range_clear(dm));
    CS_TRY(cs_prefill(m, kv, 0, prompt, prompt_len));
    CS_TRY(cs_kv_set_len(dkv, 0, 0));
    int64_t draft_rows = 0;                       // rows of the accepted sequence in the draft cache

    const int64_t stride = cs_round_up(prompt_len + max_new + kmax + 2, 4);
    int32_t* d = nullptr;
    CS_HIP(hipMalloc(&d, (size_t)(stride + 16 + (delta > 0 ? delta : 1)) * 4));
    // d_len: [0] hist_len, [1] room, [2] accepted, [3] next, [4] draft_len, [5] scratch, [6] zero
    int32_t* d_len = d + stride;
    int32_t* d_proposed = d_len + 16;             // the draft model's tokens
    int32_t init[7] = {(int32_t)prompt_len, (int32_t)max_new, 0, 0, 0, 0, 0};
    int rc = CS_OK;
    if (hipMemcpy(d, prompt, (size_t)prompt_len * 4, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(d_len, init, sizeof(init), hipMemcpyHostToDevice) != hipSuccess) {
        cs_set_error("cs_decode_merged: copy to device failed");
        rc = CS_E_DEVICE;
    }
    hipStream_t s = nullptr;
    int64_t emitted = 0, n = prompt_len;
    bool stop = false;
    // one step; returns through rc.  A lambda so that every exit path frees the buffer below.
    auto step = [&]() -> int {
        const int64_t room = max_new - emitted;
        int dl = 0;
        CS_REQUIRE(kv_max_ub(kv) + 1 + kmax + 1 <= stride, CS_E_CAPACITY, "history buffer may overflow");
        // step 1: copy opportunity
        if (k > 0) {
            CS_TRY(cs_scan_launch(d, stride, d_len, 1, gamma, k, policy, kv->scan_keys, kv_scan_slots(kv),
                                  m->match_pos, nullptr, m->draft, m->draft_len, d_len + 1, s));
            CS_HIP(hipMemcpy(&dl, m->draft_len, 4, hipMemcpyDeviceToHost));
        }
        k_pending<<<1, 64, 0, s>>>(d, stride, d_len, 1, m->pending);
        CS_TRY(cs_launch_ok("k_pending"));
        int block = 0, proposed = 0;
        const int32_t* draft_ptr = m->draft;
        const int32_t* len_ptr = d_len + 6;       // zero: a plain decode step
        if (dl > 0) {                             // step 2: verify the copied block
            block = k;
            len_ptr = m->draft_len;
        } else if (delta > 0 && room > 1) {       // step 3: the draft model proposes
            proposed = (int)(delta < room - 1 ? delta : room - 1);
            while (draft_rows < n - 1) {          // read what was accepted since it last ran
                const int64_t left = n - 1 - draft_rows;
                const int rows = (int)(left < dm->prefill_rows ? left : dm->prefill_rows);
                CS_HIP(hipMemcpyAsync(dm->tok, d + draft_rows, (size_t)rows * 4, hipMemcpyDeviceToDevice, s));
                CS_TRY(forward_layers(dm, dkv, rows, s));
                k_add_i32<<<1, 64, 0, s>>>(dkv->d_len, rows, 1);
                CS_TRY(cs_launch_ok("k_add_i32"));
                dkv->h_len_ub[0] += rows;
                draft_rows += rows;
                st.draft_forwards += 1;
            }
            for (int i = 0; i < proposed; ++i) {  // one greedy token per forward pass
                const int32_t* tok = i == 0 ? m->pending : d_proposed + i - 1;
                CS_TRY(verify_impl(dm, dkv, tok, nullptr, d_len + 6, 0, d_len + 5, d_proposed + i, nullptr,
                                   nullptr, 0, nullptr, nullptr, s));
                draft_rows += 1;
                st.draft_forwards += 1;
            }
            CS_TRY(cs_fill_i32_launch(d_len + 4, proposed, 1, s));
            block = proposed;
            draft_ptr = d_proposed;
            len_ptr = d_len + 4;
        }
        CS_TRY(verify_impl(m, kv, m->pending, draft_ptr, len_ptr, block, d_len + 2, d_len + 3, nullptr, d,
                           stride, d_len, d_len + 1, s));
        int32_t h[4];
        CS_HIP(hipMemcpy(h, d_len, sizeof(h), hipMemcpyDeviceToHost));
        const int tau = h[2], got = tau + 1;
        kv->h_len_ub[0] = h[0] - 1;               // true length: everything but the pending token
        if (proposed > 0) {
            // the draft cache holds the old sequence and every proposal it was fed (all but the last)
            draft_rows = n + (tau < proposed - 1 ? tau : proposed - 1);
            CS_TRY(cs_kv_set_len(dkv, 0, draft_rows));
        }
        CS_HIP(hipMemcpy(out_tokens + emitted, d + (h[0] - got), (size_t)got * 4, hipMemcpyDeviceToHost));
        n = h[0];
        st.steps += 1;
        if (dl > 0) { st.copy_attempts += 1; st.copy_drafted += dl; st.copy_accepted += tau; }
        if (proposed > 0) { st.spec_attempts += 1; st.spec_drafted += proposed; st.spec_accepted += tau; }
        for (int i = 0; i < got; ++i) {
            if (eos_id >= 0 && out_tokens[emitted + i] == eos_id) {
                emitted += i + 1;
                stop = true;
                return CS_OK;
            }
        }
        emitted += got;
        return CS_OK;
    };
    while (rc == CS_OK && emitted < max_new && !stop) rc = step();
    (void)hipFree(d);
    if (rc != CS_OK) return rc;
    *n_out = emitted;
    if (stats) *stats = st;
    CS_TRY(range_check_after_loop(dm, "cs_decode_merged (draft model)"));
    return range_check_after_loop(m, "cs_decode_merged");
}

// -------------------------------------------------------------------------------------
// single operations
// -------------------------------------------------------------------------------------
extern "C" int cs_op_gemm(cs_model* m, int32_t dtype, const void* X, const void* W, float* Y, int32_t R,
                          int32_t N, int32_t K, void* stream) {
    CS_REQUIRE(m && X && W && Y, CS_E_ARG, "cs_op_gemm: NULL argument");
    CS_REQUIRE(R >= 0 && N >= 1 && K >= 1, CS_E_ARG, "cs_op_gemm: bad shape");
    hipStream_t s = (hipStream_t)stream;
    if (R == 0) return CS_OK;
    if (dtype == CS_F32) return cs_gemm_plain_launch(CS_F32, (const float*)X, W, Y, R, N, K, s);
    CS_REQUIRE(dtype == CS_BF16, CS_E_ARG, "cs_op_gemm: bad dtype");
    CS_REQUIRE(m->fast, CS_E_STATE, "cs_op_gemm(bf16) needs a model that runs the bf16 kernels");
    // the tuned kernel reads W in its tiled fp16 layout and X as fp16: convert into temporaries
    void* wt = nullptr;
    const size_t x_bytes = cs_xt_bytes(R, K);
    CS_HIP(hipMalloc(&wt, (size_t)N * K * 2 + 2 * x_bytes));
    void* xt = (char*)wt + (size_t)N * K * 2;
    int rc = cs_tile_weights_launch(W, nullptr, N, K, 0, N, 0, wt, nullptr, s);
    if (rc == CS_OK) rc = cs_convert_launch(X, CS_T_BF16, xt, CS_T_F16, (int64_t)R * K, s);
    X = xt;
    if (rc == CS_OK && cs_gemm_x_tiled(R, N)) {            // the many-row kernel reads fragment order
        void* xt2 = (char*)xt + x_bytes;
        rc = cs_tile_x_launch(xt, xt2, R, K, s);
        X = xt2;
    }
    int np = 1;
    if (rc == CS_OK) {
        if ((size_t)R * N > m->part_floats) {   // too large for the workspace: no K split
            rc = cs_gemm_launch(m, X, wt, Y, R, N, K, CS_GEMM_STORE, 0, nullptr, s);
        } else {
            rc = cs_gemm_launch(m, X, wt, m->part, R, N, K, CS_GEMM_STORE, 1, &np, s);
            if (rc == CS_OK) {
                const int64_t n = (int64_t)R * N;
                k_sum_parts<<<(unsigned)(cs_ceil_div(n, 256) < 2048 ? cs_ceil_div(n, 256) : 2048), 256, 0,
                              s>>>(m->part, np, n, Y);
                rc = cs_launch_ok("k_sum_parts");
            }
        }
    }
    if (hipStreamSynchronize(s) != hipSuccess && rc == CS_OK) {
        cs_set_error("cs_op_gemm: synchronize failed");
        rc = CS_E_DEVICE;
    }
    (void)hipFree(wt);
    return rc;
}

extern "C" int cs_op_attention(cs_model* m, cs_kv* kv, int32_t layer, const float* q, int32_t rows,
                               float* out, void* stream) {
    CS_REQUIRE(m && kv && q && out, CS_E_ARG, "cs_op_attention: NULL argument");
    CS_REQUIRE(kv->m == m, CS_E_STATE, "kv cache belongs to a different model");
    CS_REQUIRE(layer >= 0 && layer < m->cfg.n_layers, CS_E_ARG, "layer out of range");
    CS_REQUIRE(rows >= 1 && rows <= m->rows_max, CS_E_ARG, "rows outside 1..max_k+1");
    hipStream_t s = (hipStream_t)stream;
    CS_TRY(kv_check_room(kv, rows));
    const int64_t n = (int64_t)kv->B * rows * m->cfg.n_heads * m->cfg.head_dim;
    CS_TRY(cs_convert_launch(q, CS_T_F32, m->q, m->fast ? CS_T_BF16 : CS_T_F32, n, s));
    CS_TRY(cs_attention_launch(m, kv, layer, rows, kv_max_ub(kv), 0, nullptr, 0, s));
    return cs_convert_launch(m->xn, m->fast ? CS_T_F16 : CS_T_F32, out, CS_T_F32, n, s);
}

extern "C" int cs_op_argmax_accept(cs_model* m, const float* logits, int32_t B, int32_t k, int32_t V,
                                   const int32_t* draft, const int32_t* draft_len,
                                   int32_t* accepted_len, int32_t* next_token, int32_t* row_argmax,
                                   void* stream) {
    CS_REQUIRE(m && logits && draft_len && accepted_len && next_token && (draft || k == 0), CS_E_ARG,
               "cs_op_argmax_accept: NULL argument");
    CS_REQUIRE(B >= 1 && k >= 0 && V >= 1 && B * (k + 1) <= m->R_max, CS_E_ARG,
               "cs_op_argmax_accept: B*(k+1) exceeds the model's max_batch*(max_k+1)");
    return cs_argmax_accept_launch(m, logits, B, k, V, draft, draft_len, accepted_len, next_token,
                                   row_argmax, nullptr, nullptr, 0, nullptr, nullptr,
                                   (hipStream_t)stream);
}
