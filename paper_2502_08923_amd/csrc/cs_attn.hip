// Block attention of the verify pass: the k+1 block rows of every stream attend to the
// stream's KV cache plus the causal part of the block itself (Sec. 3.2: the draft is
// appended to the context and evaluated in one pass; App. B.2: per-layer K, V).
//
// The pass is bound by streaming K and V from HBM once.  All G*(k+1) query rows that share
// a KV head (G = n_heads / n_kv_heads) are processed together, so each K/V byte is used
// G*(k+1) times: 44 flop per byte at k = 10, more than the vector ALUs can deliver at
// 8 TB/s, which is why QK^T and PV run on the matrix cores although the kernel is graded
// against the HBM roofline.
//
// Tuned kernel, per wave (no LDS, everything stays in registers):
//   S^T[token][qrow] = K[token][:] . Q[qrow][:]        v_mfma_f32_16x16x32_bf16, A = K rows
//   O^T[hd][qrow]   += V^T[hd][token] * P^T[token][qrow]                         A = V^T rows
// K rows are fed in a permuted token order chosen so that the S^T accumulator layout of two
// 16-token tiles is exactly the B-operand layout of the PV product (8 consecutive tokens per
// lane); V is cached transposed (token index contiguous) so its A operand is one 16-byte
// load per lane.  Softmax runs online in float32 (base 2), the row maximum is shared by the
// four lanes that hold a query row, and O is only rescaled when some maximum moved.
// The token range of a stream is split over waves; a merge kernel combines the partial
// (max, sum, O) triples.
#include "cs_common.h"

// -------------------------------------------------------------------------------------
// plain reference kernel: one workgroup per (block row, query head, stream)
// -------------------------------------------------------------------------------------
#define PA_THREADS 256
#define PA_CHUNK 2048

__device__ __forceinline__ float block_max(float v, float* wred) {
    v = cs_wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) wred[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = wred[0];
    for (int w = 1; w < PA_THREADS / CS_WAVE; ++w) r = fmaxf(r, wred[w]);
    return r;
}
__device__ __forceinline__ float block_sum(float v, float* wred) {
    v = cs_wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) wred[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = 0.f;
    for (int w = 0; w < PA_THREADS / CS_WAVE; ++w) r += wred[w];
    return r;
}

template <typename WT, typename QT, typename OT>
__global__ __launch_bounds__(PA_THREADS) void k_attn_plain(const QT* __restrict__ q,
                                                           const WT* __restrict__ kc,
                                                           const WT* __restrict__ vc,
                                                           const int32_t* __restrict__ kv_len,
                                                           int rows, int H, int KVH, int hd,
                                                           int64_t cap, OT* __restrict__ out) {
    __shared__ float sq[256];
    __shared__ float sc[PA_CHUNK];
    __shared__ float red[PA_THREADS];
    __shared__ float wred[PA_THREADS / CS_WAVE];
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x;
    const int r = b * rows + i;
    const int g = h / (H / KVH);
    const int n_ctx = kv_len[b] + i + 1;
    const WT* __restrict__ K = kc + ((int64_t)b * KVH + g) * cap * hd;
    const WT* __restrict__ V = vc + ((int64_t)b * KVH + g) * hd * cap;
    if (tid < hd) sq[tid] = cs_ld(q, ((int64_t)r * H + h) * hd + tid);
    __syncthreads();
    const float scale = 1.0f / sqrtf((float)hd);
    const int d = tid % hd, part = tid / hd, nparts = PA_THREADS / hd;
    float m_run = -INFINITY, l_run = 0.f, o = 0.f;
    for (int c0 = 0; c0 < n_ctx; c0 += PA_CHUNK) {
        const int cn = min(PA_CHUNK, n_ctx - c0);
        float lmax = -INFINITY;
        for (int t = tid; t < cn; t += PA_THREADS) {
            const WT* __restrict__ kr = K + (int64_t)(c0 + t) * hd;
            float s = 0.f;
            for (int e = 0; e < hd; ++e) s += sq[e] * cs_ld(kr, e);
            s *= scale;
            sc[t] = s;
            lmax = fmaxf(lmax, s);
        }
        const float mc = block_max(lmax, wred);
        const float m_new = fmaxf(m_run, mc);
        const float alpha = expf(m_run - m_new);
        float lsum = 0.f;
        for (int t = tid; t < cn; t += PA_THREADS) {
            const float p = expf(sc[t] - m_new);
            sc[t] = p;
            lsum += p;
        }
        const float lc = block_sum(lsum, wred);   // its barriers also publish sc[]
        l_run = l_run * alpha + lc;
        float acc = 0.f;
        const WT* __restrict__ vr = V + (int64_t)d * cap + c0;
        for (int t = part; t < cn; t += nparts) acc += sc[t] * cs_ld(vr, t);
        o = o * alpha + acc;
        m_run = m_new;
        __syncthreads();
    }
    red[tid] = o;
    __syncthreads();
    if (part == 0) {
        float tot = 0.f;
        for (int p = 0; p < nparts; ++p) tot += red[p * hd + d];
        cs_st(out, ((int64_t)r * H + h) * hd + d, tot / l_run);
    }
}

// -------------------------------------------------------------------------------------
// tuned bf16 kernel
// -------------------------------------------------------------------------------------
#define FA_NT 3            // 16-row query tiles per wave  (48 query rows)
#define FA_QROWS (16 * FA_NT)

// Partial layout: po[item][wave][qrow][HD] float, pml[item][wave][qrow][2] = (max2, sum)
// where item = (b*KVH + kvh)*nqg + qg and max2 is in base-2 scaled units.
template <int HD>
__global__ __launch_bounds__(256) void k_attn_mfma(const bf16_t* __restrict__ q,
                                                   const bf16_t* __restrict__ kc,
                                                   const bf16_t* __restrict__ vc,
                                                   const int32_t* __restrict__ kv_len, int rows,
                                                   int H, int KVH, int64_t cap, int Tw, int nqg,
                                                   int nwaves, float* __restrict__ po,
                                                   float* __restrict__ pml) {
    constexpr int KS = HD / 32;      // MFMA k-steps over the head dimension
    constexpr int MT = HD / 16;      // 16-row tiles of O^T
    constexpr int HQ = HD / 4;       // head-dim elements per lane group
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int qg = blockIdx.x % nqg;
    const int wg = (blockIdx.x / nqg) * 4 + wave;       // wave index along the token axis
    const int kvh = blockIdx.y, b = blockIdx.z;
    const int G = H / KVH;
    const int QR = G * rows;
    const int L = kv_len[b];
    const int n_tok = L + rows;
    const int t_begin = wg * Tw;
    if (t_begin >= n_tok) return;                       // merge kernel skips these waves too
    const int t_end = min(n_tok, t_begin + Tw);
    const bf16_t* __restrict__ K = kc + ((int64_t)b * KVH + kvh) * cap * HD;
    const bf16_t* __restrict__ V = vc + ((int64_t)b * KVH + kvh) * HD * cap;

    // query rows of this wave: global qrow n = qg*48 + nt*16 + c  <->  block row n / G, head n % G
    bf16x8 qb[FA_NT][KS];
    int qi[FA_NT];               // block row index of the lane's query row (for the causal mask)
#pragma unroll
    for (int nt = 0; nt < FA_NT; ++nt) {
        const int n = qg * FA_QROWS + nt * 16 + c;
        const bool ok = n < QR;
        const int i = ok ? n / G : 0, gq = ok ? n % G : 0;
        qi[nt] = ok ? i : -1;
        const bf16_t* qp = q + (((int64_t)(b * rows + i)) * H + kvh * G + gq) * HD + g * HQ;
#pragma unroll
        for (int s = 0; s < KS; ++s)
            qb[nt][s] = ok ? *reinterpret_cast<const bf16x8*>(qp + s * 8)
                           : (bf16x8){0, 0, 0, 0, 0, 0, 0, 0};
    }

    f32x4 oacc[MT][FA_NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < FA_NT; ++nt) oacc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float m_run[FA_NT], l_lane[FA_NT];
#pragma unroll
    for (int nt = 0; nt < FA_NT; ++nt) { m_run[nt] = -INFINITY; l_lane[nt] = 0.f; }

    const float scale2 = 1.4426950408889634f / sqrtf((float)HD);

    // K tile a, MFMA row m=c  <->  token t0 + 8*(c/4) + 4a + c%4
    const int ktok0 = 8 * (c >> 2) + (c & 3);
    bf16x8 kn[2][KS], vn[MT];
    auto load_kv = [&](int t0) {
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            const bf16_t* kp = K + (int64_t)(t0 + ktok0 + 4 * a) * HD + g * HQ;
#pragma unroll
            for (int s = 0; s < KS; ++s) kn[a][s] = *reinterpret_cast<const bf16x8*>(kp + s * 8);
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            vn[mt] = *reinterpret_cast<const bf16x8*>(V + (int64_t)(mt * 16 + c) * cap + t0 + 8 * g);
    };

    load_kv(t_begin);
    for (int t0 = t_begin; t0 < t_end; t0 += 32) {
        bf16x8 kr[2][KS], vr[MT];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int s = 0; s < KS; ++s) kr[a][s] = kn[a][s];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) vr[mt] = vn[mt];
        if (t0 + 32 < t_end) load_kv(t0 + 32);

        // scores: lane (c, g) gets tokens t0 + 8g + (4a + j) of query row nt*16 + c
        f32x4 sacc[2][FA_NT];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int nt = 0; nt < FA_NT; ++nt) {
                f32x4 z = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < KS; ++s)
                    z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kr[a][s], qb[nt][s], z, 0, 0, 0);
                sacc[a][nt] = z;
            }
        const bool tail = t0 + 32 > L;       // block touches the new rows or the dead region
        if (tail) {
            // dead cache rows may hold anything: zero their V so that 0 * garbage stays 0
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (t0 + 8 * g + j >= n_tok) vr[mt][j] = (bf16_t)0.f;
        }
        bool moved = false;
        float alpha[FA_NT];
        bf16x8 pb[FA_NT];
#pragma unroll
        for (int nt = 0; nt < FA_NT; ++nt) {
            float sv[8];
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float s = sacc[a][nt][j] * scale2;
                    if (tail && (t0 + 8 * g + 4 * a + j > L + qi[nt])) s = -INFINITY;
                    sv[4 * a + j] = s;
                }
            float mx = sv[0];
#pragma unroll
            for (int j = 1; j < 8; ++j) mx = fmaxf(mx, sv[j]);
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run[nt], mx);
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
            alpha[nt] = __builtin_amdgcn_exp2f(m_run[nt] - m_safe);
            moved |= (m_new > m_run[nt]);
            m_run[nt] = m_new;
            float ls = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float p = __builtin_amdgcn_exp2f(sv[j] - m_safe);
                ls += p;
                pb[nt][j] = (bf16_t)p;
            }
            l_lane[nt] = l_lane[nt] * alpha[nt] + ls;
        }
        if (__any(moved)) {
#pragma unroll
            for (int nt = 0; nt < FA_NT; ++nt)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) oacc[mt][nt] *= alpha[nt];
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < FA_NT; ++nt)
                oacc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vr[mt], pb[nt], oacc[mt][nt], 0, 0, 0);
    }

    // partial result of this wave
    const int64_t item = ((int64_t)b * KVH + kvh) * nqg + qg;
    float* __restrict__ o_out = po + (item * nwaves + wg) * FA_QROWS * HD;
    float* __restrict__ ml_out = pml + (item * nwaves + wg) * FA_QROWS * 2;
#pragma unroll
    for (int nt = 0; nt < FA_NT; ++nt) {
        float l = l_lane[nt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        const int n = nt * 16 + c;
        if (g == 0) { ml_out[n * 2] = m_run[nt]; ml_out[n * 2 + 1] = l; }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            *reinterpret_cast<f32x4*>(o_out + (int64_t)n * HD + mt * 16 + 4 * g) = oacc[mt][nt];
    }
}

// out[r][h*HD + d] = sum_w 2^(m_w - M) O_w[d] / sum_w 2^(m_w - M) l_w
template <typename OT>
__global__ void k_attn_merge(const float* __restrict__ po, const float* __restrict__ pml,
                             const int32_t* __restrict__ kv_len, int rows, int H, int KVH, int HD,
                             int Tw, int nqg, int nwaves, OT* __restrict__ out) {
    const int n = blockIdx.x;                 // query row within the KV head: i*G + gq
    const int kvh = blockIdx.y, b = blockIdx.z;
    const int G = H / KVH;
    const int i = n / G, gq = n % G;
    const int qg = n / FA_QROWS, nl = n % FA_QROWS;
    const int n_tok = kv_len[b] + rows;
    const int nvalid = min(nwaves, (n_tok + Tw - 1) / Tw);
    const int64_t item = ((int64_t)b * KVH + kvh) * nqg + qg;
    const float* __restrict__ ml = pml + item * nwaves * FA_QROWS * 2;
    const float* __restrict__ o = po + item * nwaves * FA_QROWS * HD;
    float M = -INFINITY;
    for (int w = 0; w < nvalid; ++w) M = fmaxf(M, ml[((int64_t)w * FA_QROWS + nl) * 2]);
    for (int d = threadIdx.x; d < HD; d += blockDim.x) {
        float num = 0.f, den = 0.f;
        for (int w = 0; w < nvalid; ++w) {
            const float mw = ml[((int64_t)w * FA_QROWS + nl) * 2];
            if (mw == -INFINITY) continue;
            const float sc = __builtin_amdgcn_exp2f(mw - M);
            den += sc * ml[((int64_t)w * FA_QROWS + nl) * 2 + 1];
            num += sc * o[((int64_t)w * FA_QROWS + nl) * HD + d];
        }
        const int r = b * rows + i;
        cs_st(out, ((int64_t)r * H + kvh * G + gq) * HD + d, num / den);
    }
}

int cs_attention_launch(const cs_model* m, cs_kv* kv, int layer, int rows, int64_t len_ub,
                        hipStream_t s) {
    const cs_model_cfg& c = m->cfg;
    const int B = kv->B, H = c.n_heads, KVH = c.n_kv_heads, hd = c.head_dim;
    const int64_t per_layer = (int64_t)B * KVH * kv->cap * hd;
    if (!m->fast) {
        dim3 grid(rows, H, B);
        if (c.dtype == CS_BF16)
            k_attn_plain<bf16_t, float, float><<<grid, PA_THREADS, 0, s>>>(
                (const float*)m->q, (const bf16_t*)kv->k + layer * per_layer,
                (const bf16_t*)kv->v + layer * per_layer, kv->d_len, rows, H, KVH, hd, kv->cap,
                (float*)m->xn);
        else
            k_attn_plain<float, float, float><<<grid, PA_THREADS, 0, s>>>(
                (const float*)m->q, (const float*)kv->k + layer * per_layer,
                (const float*)kv->v + layer * per_layer, kv->d_len, rows, H, KVH, hd, kv->cap,
                (float*)m->xn);
        return cs_launch_ok("k_attn_plain");
    }
    const int G = H / KVH;
    const int QR = G * rows;
    const int nqg = (int)cs_ceil_div(QR, FA_QROWS);
    const int64_t n_tok_ub = len_ub + rows;
    // about two workgroups per compute unit, at least 128 tokens per wave
    int nsplit = (int)cs_ceil_div(512, (int64_t)B * KVH * nqg);
    const int max_split = (int)cs_ceil_div(n_tok_ub, 4 * 128);
    if (nsplit > max_split) nsplit = max_split;
    if (nsplit < 1) nsplit = 1;
    int Tw = (int)cs_round_up(cs_ceil_div(n_tok_ub, (int64_t)nsplit * 4), 32);
    int nwaves = (int)cs_ceil_div(n_tok_ub, Tw);
    nsplit = (int)cs_ceil_div(nwaves, 4);
    nwaves = nsplit * 4;
    const size_t need = (size_t)B * KVH * nqg * nwaves * FA_QROWS * (hd + 2);
    CS_REQUIRE(need <= m->attn_part_floats, CS_E_CAPACITY,
               "attention workspace too small (%zu > %zu floats)", need, m->attn_part_floats);
    float* po = m->attn_part;
    float* pml = m->attn_part + (size_t)B * KVH * nqg * nwaves * FA_QROWS * hd;
    const bf16_t* kc = (const bf16_t*)kv->k + layer * per_layer;
    const bf16_t* vc = (const bf16_t*)kv->v + layer * per_layer;
    dim3 grid(nsplit * nqg, KVH, B);
    const int pa = cs_prof_begin(CS_PROF_ATTN, s);
    if (hd == 128)
        k_attn_mfma<128><<<grid, 256, 0, s>>>((const bf16_t*)m->q, kc, vc, kv->d_len, rows, H, KVH,
                                              kv->cap, Tw, nqg, nwaves, po, pml);
    else
        k_attn_mfma<64><<<grid, 256, 0, s>>>((const bf16_t*)m->q, kc, vc, kv->d_len, rows, H, KVH,
                                             kv->cap, Tw, nqg, nwaves, po, pml);
    cs_prof_end(pa, s);
    CS_TRY(cs_launch_ok("k_attn_mfma"));
    dim3 mgrid(QR, KVH, B);
    const int pm = cs_prof_begin(CS_PROF_ATTN_MERGE, s);
    k_attn_merge<bf16_t><<<mgrid, hd < 64 ? 64 : hd, 0, s>>>(po, pml, kv->d_len, rows, H, KVH, hd, Tw,
                                                           nqg, nwaves, (bf16_t*)m->xn);
    cs_prof_end(pm, s);
    return cs_launch_ok("k_attn_merge");
}
