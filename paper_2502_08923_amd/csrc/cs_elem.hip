// Small kernels of the verify pass: block tokens + rotary table, embedding gather,
// residual-add + RMSNorm, rotary + KV append, SwiGLU, greedy argmax + accept rule + KV
// length update + history append (Sec. 3.2, App. B.2, App. B.3 step 2).
#include "cs_common.h"
#include <type_traits>

// -------------------------------------------------------------------------------------
// block tokens and rotary table
//   row r = b*(k+1) + i : token = pending[b] (i == 0) or draft[b][i-1] (i <= draft_len[b])
//   rope[r][j] = (cos, sin)(pos * theta^(-2j/hd)),  pos = kv_len[b] + i, in float64
// -------------------------------------------------------------------------------------
__global__ void k_tokens(const int32_t* __restrict__ pending, const int32_t* __restrict__ draft,
                         const int32_t* __restrict__ draft_len, int k, int V,
                         int32_t* __restrict__ tok) {
    const int b = blockIdx.x;
    const int rows = k + 1;
    for (int i = threadIdx.x; i < rows; i += blockDim.x) {
        int t = 0;
        if (i == 0) t = pending[b];
        else if (i - 1 < draft_len[b]) t = draft[(int64_t)b * k + i - 1];
        if (t < 0 || t >= V) t = 0;   // an out-of-vocabulary draft can never be accepted
        tok[b * rows + i] = t;
    }
}

__global__ void k_rope_table(const int32_t* __restrict__ kv_len, int rows, int half, int hd,
                             double theta, const double* __restrict__ inv_freq,
                             float2* __restrict__ rope) {
    const int r = blockIdx.x;
    const int b = r / rows, i = r % rows;
    const double pos = (double)(kv_len[b] + i);
    for (int j = threadIdx.x; j < half; j += blockDim.x) {
        const double inv = inv_freq ? inv_freq[j] : pow(theta, -2.0 * (double)j / (double)hd);
        double sn, cs;
        sincos(pos * inv, &sn, &cs);
        rope[(int64_t)r * half + j] = make_float2((float)cs, (float)sn);
    }
}

// -------------------------------------------------------------------------------------
// embedding gather: x[r][:] = embed[tok[r]][:]
// -------------------------------------------------------------------------------------
template <typename WT>
__global__ void k_embed(const WT* __restrict__ embed, const int32_t* __restrict__ tok, int d,
                        float* __restrict__ x) {
    const int r = blockIdx.x;
    const WT* __restrict__ e = embed + (int64_t)tok[r] * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) x[(int64_t)r * d + c] = cs_ld(e, c);
}

// -------------------------------------------------------------------------------------
// x[r] += sum_p part[p][r][:]   then   xn[r] = x[r] * rsqrt(mean(x[r]^2) + eps) * gain
// The split-K partial tiles of the preceding projection are reduced here, in a fixed
// order, so the result does not depend on scheduling.
// -------------------------------------------------------------------------------------
#define NORM_THREADS 1024
#define NORM_MAXV 2          // float4 vectors per thread: d <= 4 * 2 * 1024
template <typename OutT>
__global__ __launch_bounds__(NORM_THREADS) void k_addnorm(float* __restrict__ x,
                                                          const float* __restrict__ part,
                                                          int nparts, int64_t part_stride, int d,
                                                          float eps, const float* __restrict__ gain,
                                                          OutT* __restrict__ xn, int tiled,
                                                          int32_t* __restrict__ flags) {
    const int r = blockIdx.x;
    const int nvec = d >> 2;                 // d is a multiple of 4 (checked on the host)
    float4 v[NORM_MAXV];
    float ss = 0.f;
#pragma unroll
    for (int u = 0; u < NORM_MAXV; ++u) {
        const int c = threadIdx.x + u * NORM_THREADS;
        v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (c < nvec) {
            const int64_t off = (int64_t)r * d + 4 * c;
            float4 a = *reinterpret_cast<const float4*>(x + off);
            // all partial tiles are fetched before the first add: the loads are independent
#pragma unroll 8
            for (int p = 0; p < nparts; ++p) {
                const float4 t = *reinterpret_cast<const float4*>(part + p * part_stride + off);
                a.x += t.x; a.y += t.y; a.z += t.z; a.w += t.w;
            }
            if (nparts > 0) *reinterpret_cast<float4*>(x + off) = a;
            v[u] = a;
            ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
        }
    }
    if (!xn) return;
    ss = cs_wave_sum(ss);
    __shared__ float wsum[NORM_THREADS / CS_WAVE];
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < NORM_THREADS / CS_WAVE; ++w) tot += wsum[w];
    const float scale = 1.0f / sqrtf(tot / (float)d + eps);
    bool hit = false;
#pragma unroll
    for (int u = 0; u < NORM_MAXV; ++u) {
        const int c = threadIdx.x + u * NORM_THREADS;
        if (c < nvec) {
            const float4 gn = *reinterpret_cast<const float4*>(gain + 4 * c);
            // tiled: the reader is the many-row GEMM, which wants fragment order
            const int64_t off = tiled ? cs_xt_index(r, 4 * c, d) : (int64_t)r * d + 4 * c;
            if constexpr (std::is_same<OutT, f16_t>::value) {   // one 8-byte store
                // the float16 input of the next projection: saturated, and reported if it was
                const f16x4 o = (f16x4){cs_f16_sat(v[u].x * scale * gn.x, hit), cs_f16_sat(v[u].y * scale * gn.y, hit),
                                        cs_f16_sat(v[u].z * scale * gn.z, hit), cs_f16_sat(v[u].w * scale * gn.w, hit)};
                *reinterpret_cast<f16x4*>(xn + off) = o;
            } else {
                cs_st(xn, off + 0, v[u].x * scale * gn.x);
                cs_st(xn, off + 1, v[u].y * scale * gn.y);
                cs_st(xn, off + 2, v[u].z * scale * gn.z);
                cs_st(xn, off + 3, v[u].w * scale * gn.w);
            }
        }
    }
    cs_range_report(flags, hit, CS_RANGE_NORM);
}

// -------------------------------------------------------------------------------------
// rotary + KV append.  qkv[r] = sum_p part[p][r][:] holds q heads, k heads, v heads.
// q -> rotated, stored [R][H][hd] (QT); k -> rotated, rounded to the cache type, stored at
// cache row kv_len[b]+i; v -> stored transposed in 128-token blocks (cs_v_index).
// -------------------------------------------------------------------------------------
template <typename WT, typename QT>
__global__ __launch_bounds__(64) void k_rope_append(const float* __restrict__ qkv, int nparts,
                                                    int64_t part_stride,
                                                    const float2* __restrict__ rope,
                                                    const int32_t* __restrict__ kv_len, int rows,
                                                    int H, int KVH, int hd, int64_t cap,
                                                    WT* __restrict__ kc, WT* __restrict__ vc,
                                                    QT* __restrict__ q,
                                                    const float* __restrict__ bias) {
    const int r = blockIdx.y, head = blockIdx.x;     // head: q heads, then k heads, then v heads
    const int b = r / rows, i = r % rows;
    const int half = hd / 2;
    const int nq = (H + 2 * KVH) * hd;
    const int64_t pos = (int64_t)kv_len[b] + i;
    for (int j = threadIdx.x; j < half; j += 64) {
        const int64_t i0 = (int64_t)r * nq + (int64_t)head * hd + j;
        float a = 0.f, c = 0.f;
#pragma unroll 8
        for (int p = 0; p < nparts; ++p) {
            a += qkv[p * part_stride + i0];
            c += qkv[p * part_stride + i0 + half];
        }
        if (bias) {                                   // projection bias, before the rotation
            a += bias[head * hd + j];
            c += bias[head * hd + j + half];
        }
        if (head < H + KVH) {
            const float2 cs = rope[(int64_t)r * half + j];
            const float ra = a * cs.x - c * cs.y;
            const float rc = c * cs.x + a * cs.y;
            a = ra; c = rc;
        }
        if (head < H) {
            cs_st(q, ((int64_t)r * H + head) * hd + j, a);
            cs_st(q, ((int64_t)r * H + head) * hd + j + half, c);
        } else if (head < H + KVH) {
            const int g = head - H;
            WT* __restrict__ row = kc + (((int64_t)b * KVH + g) * cap + pos) * hd;
            cs_st(row, j, a);
            cs_st(row, j + half, c);
        } else {
            const int g = head - H - KVH;
            WT* __restrict__ base = vc + ((int64_t)b * KVH + g) * hd * cap;
            cs_st(base, cs_v_index(pos, j, hd), a);
            cs_st(base, cs_v_index(pos, j + half, hd), c);
        }
    }
}

// The same for blocks of many rows (wide verify blocks, prompt blocks), bf16 cache and queries:
// a workgroup takes RA_ROWS consecutive block rows of one head, every thread four adjacent
// elements of both rotary halves (16-byte loads of the partial tiles, 8-byte stores), and the V
// rows, whose cache keeps the token index contiguous (cs_v_index), go through an LDS tile so that
// the rows of a workgroup are written as runs of consecutive tokens instead of one element per line.
#define RA_ROWS 32
#define RA_THREADS 256
__global__ __launch_bounds__(RA_THREADS) void k_rope_append_rows(
    const float* __restrict__ qkv, int nparts, int64_t part_stride, const float2* __restrict__ rope,
    const int32_t* __restrict__ kv_len, int rows, int R, int H, int KVH, int hd, int64_t cap,
    bf16_t* __restrict__ kc, bf16_t* __restrict__ vc, bf16_t* __restrict__ q,
    const float* __restrict__ bias) {
    __shared__ bf16_t vt[256][RA_ROWS + 2];            // [d][row of the workgroup], hd <= 256
    __shared__ int64_t voff[RA_ROWS];                  // cache offset of each row's token (v heads)
    const int head = blockIdx.x;                       // q heads, then k heads, then v heads
    const int rr = threadIdx.x >> 3, t8 = threadIdx.x & 7;
    const int r = blockIdx.y * RA_ROWS + rr;
    const int half = hd / 2;
    const int nq = (H + 2 * KVH) * hd;
    const bool live = r < R;
    const int b = live ? r / rows : 0, i = live ? r % rows : 0;
    const int64_t pos = live ? (int64_t)kv_len[b] + i : 0;
    const bool is_v = head >= H + KVH;
    if (is_v && t8 == 0) voff[rr] = live ? ((int64_t)b * KVH + (head - H - KVH)) * hd * cap + cs_v_index(pos, 0, hd) : -1;
    if (live) {
        for (int j = t8 * 4; j < half; j += 32) {
            const int64_t i0 = (int64_t)r * nq + (int64_t)head * hd + j;
            f32x4 a = (f32x4){0.f, 0.f, 0.f, 0.f}, c = a;
            for (int p = 0; p < nparts; ++p) {         // in order: the same sums as the other kernels
                a += *reinterpret_cast<const f32x4*>(qkv + p * part_stride + i0);
                c += *reinterpret_cast<const f32x4*>(qkv + p * part_stride + i0 + half);
            }
            if (bias) {                               // projection bias, before the rotation
                a += *reinterpret_cast<const f32x4*>(bias + head * hd + j);
                c += *reinterpret_cast<const f32x4*>(bias + head * hd + j + half);
            }
            if (!is_v) {
                const f32x4 cs0 = *reinterpret_cast<const f32x4*>(rope + (int64_t)r * half + j);
                const f32x4 cs1 = *reinterpret_cast<const f32x4*>(rope + (int64_t)r * half + j + 2);
                const f32x4 co = (f32x4){cs0[0], cs0[2], cs1[0], cs1[2]};
                const f32x4 si = (f32x4){cs0[1], cs0[3], cs1[1], cs1[3]};
                const f32x4 ra = a * co - c * si;
                const f32x4 rc = c * co + a * si;
                a = ra;
                c = rc;
            }
            bf16x4 oa, oc;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                oa[u] = (bf16_t)a[u];
                oc[u] = (bf16_t)c[u];
            }
            if (head < H) {
                bf16_t* dst = q + ((int64_t)r * H + head) * hd + j;
                *reinterpret_cast<bf16x4*>(dst) = oa;
                *reinterpret_cast<bf16x4*>(dst + half) = oc;
            } else if (!is_v) {
                bf16_t* dst = kc + (((int64_t)b * KVH + (head - H)) * cap + pos) * hd + j;
                *reinterpret_cast<bf16x4*>(dst) = oa;
                *reinterpret_cast<bf16x4*>(dst + half) = oc;
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    vt[j + u][rr] = oa[u];
                    vt[j + half + u][rr] = oc[u];
                }
            }
        }
    }
    if (!is_v) return;                                 // uniform over the workgroup
    __syncthreads();
    // lane -> token of the workgroup, wave and step -> d: a wave writes 2 runs of 32 tokens
    const int tok = threadIdx.x & (RA_ROWS - 1);
    const int64_t off = voff[tok];
    if (off < 0) return;
    for (int d = threadIdx.x / RA_ROWS; d < hd; d += RA_THREADS / RA_ROWS) vc[off + (int64_t)d * CS_VBLK] = vt[d][tok];
}

// -------------------------------------------------------------------------------------
// SwiGLU on the interleaved gate/up projection (plain path): row layout of gu matches the
// packed weight: index (f/16)*32 + 16*u + f%16.
// -------------------------------------------------------------------------------------
template <typename AT>
__global__ void k_swiglu(const float* __restrict__ gu, int F, AT* __restrict__ act) {
    const int r = blockIdx.y;
    const int f = blockIdx.x * blockDim.x + threadIdx.x;
    if (f >= F) return;
    const int64_t base = (int64_t)r * 2 * F + (f / 16) * 32 + (f % 16);
    const float g = gu[base], u = gu[base + 16];
    cs_st(act, (int64_t)r * F + f, g / (1.0f + expf(-g)) * u);
}

// -------------------------------------------------------------------------------------
// greedy argmax (lowest index on ties) in two stages + accept rule + state update
// -------------------------------------------------------------------------------------
#define AM_THREADS 256
__device__ __forceinline__ void am_take(float& bv, int& bi, float v, int i) { cs_am_take(bv, bi, v, i); }

__global__ __launch_bounds__(AM_THREADS) void k_argmax_partial(const float* __restrict__ logits,
                                                               int V, int Vc, int vec_ok,
                                                               int32_t* __restrict__ out) {
    const int r = blockIdx.y, c = blockIdx.x, nch = gridDim.x;
    const float* __restrict__ row = logits + (int64_t)r * V;
    const int lo = c * Vc, hi = min(V, lo + Vc);
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    if (vec_ok) {
        // four independent 16-byte loads per thread are issued before any of them is compared,
        // so a workgroup keeps 16 KB in flight; candidates are visited in increasing index order
        // per thread, which keeps "first index on ties" a plain strict comparison
        int i = lo + (int)threadIdx.x * 4;
        for (; i + 3 * AM_THREADS * 4 + 3 < hi; i += 4 * AM_THREADS * 4) {
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4*>(row + i + u * AM_THREADS * 4);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int iu = i + u * AM_THREADS * 4;
                if (v[u].x > bv) { bv = v[u].x; bi = iu; }
                if (v[u].y > bv) { bv = v[u].y; bi = iu + 1; }
                if (v[u].z > bv) { bv = v[u].z; bi = iu + 2; }
                if (v[u].w > bv) { bv = v[u].w; bi = iu + 3; }
            }
        }
        for (; i < hi; i += AM_THREADS * 4) {
            if (i + 3 < hi) {
                const float4 v = *reinterpret_cast<const float4*>(row + i);
                if (v.x > bv) { bv = v.x; bi = i; }
                if (v.y > bv) { bv = v.y; bi = i + 1; }
                if (v.z > bv) { bv = v.z; bi = i + 2; }
                if (v.w > bv) { bv = v.w; bi = i + 3; }
            } else {
                for (int u = i; u < hi; ++u)
                    if (row[u] > bv) { bv = row[u]; bi = u; }
            }
        }
    } else {
        for (int i = lo + (int)threadIdx.x; i < hi; i += AM_THREADS)
            if (row[i] > bv) { bv = row[i]; bi = i; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        am_take(bv, bi, ov, oi);
    }
    __shared__ float sv[AM_THREADS / CS_WAVE];
    __shared__ int si[AM_THREADS / CS_WAVE];
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < AM_THREADS / CS_WAVE; ++w) am_take(bv, bi, sv[w], si[w]);
        out[((int64_t)r * nch + c) * 2] = __float_as_int(bv);
        out[((int64_t)r * nch + c) * 2 + 1] = bi;
    }
}

// One workgroup per stream.  a_i = argmax of row i; tau = leading agreement with the draft;
// (a stream whose emission budget `room` is used up is skipped, see below)
// next = a_tau; the KV length grows by tau+1 (App. B.2: truncation past the accepted rows);
// the accepted drafts and the free token are appended to the history (App. B.3 step 2d).
// The four waves share the rows; a wave reduces the nch partial pairs of a row (up to one per
// 128 vocabulary entries when the lm_head produced them itself) with four loads in flight per lane.
#define ACC_THREADS 256
__global__ __launch_bounds__(ACC_THREADS) void k_accept(const int32_t* __restrict__ part, int nch, int k,
                                                        const int32_t* __restrict__ draft,
                                                        const int32_t* __restrict__ draft_len,
                                                        int32_t* __restrict__ accepted,
                                                        int32_t* __restrict__ next_tok,
                                                        int32_t* __restrict__ row_argmax,
                                                        int32_t* __restrict__ row_argmax_out,
                                                        int32_t* __restrict__ kv_len,
                                                        int32_t* __restrict__ hist, int64_t hist_stride,
                                                        int32_t* __restrict__ hist_len,
                                                        int32_t* __restrict__ room) {
    const int b = blockIdx.x;
    const int rows = k + 1;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = wave; i < rows; i += ACC_THREADS / 64) {
        const int r = b * rows + i;
        const int2* __restrict__ p = reinterpret_cast<const int2*>(part) + (int64_t)r * nch;
        float bv = -INFINITY;
        int bi = 0x7fffffff;
        for (int c0 = 0; c0 < nch; c0 += 256) {
            int2 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + lane + 64 * u;
                v[u] = c < nch ? p[c] : make_int2(__float_as_int(-INFINITY), 0x7fffffff);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) am_take(bv, bi, __int_as_float(v[u].x), v[u].y);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float ov = __shfl_xor(bv, o, 64);
            const int oi = __shfl_xor(bi, o, 64);
            am_take(bv, bi, ov, oi);
        }
        if (lane == 0) {
            if (bi == 0x7fffffff) bi = 0;
            row_argmax[r] = bi;
            if (row_argmax_out) row_argmax_out[r] = bi;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (room && room[b] <= 0) {
            // a stream with no emission budget left takes no part: nothing is accepted,
            // emitted or appended, and its cache length stays (the row it computed is dead)
            accepted[b] = 0;
            next_tok[b] = -1;
            return;
        }
        const int m = min(draft_len[b], k);
        int tau = 0;
        while (tau < m && row_argmax[b * rows + tau] == draft[(int64_t)b * k + tau]) ++tau;
        const int nxt = row_argmax[b * rows + tau];
        accepted[b] = tau;
        next_tok[b] = nxt;
        if (kv_len) kv_len[b] += tau + 1;
        if (hist) {
            const int n = hist_len[b];
            int32_t* __restrict__ h = hist + (int64_t)b * hist_stride;
            for (int i = 0; i < tau; ++i) h[n + i] = draft[(int64_t)b * k + i];
            h[n + tau] = nxt;
            hist_len[b] = n + tau + 1;
            if (room) room[b] -= tau + 1;
        }
    }
}

template <typename S, typename D>
__global__ void k_convert(const S* __restrict__ src, D* __restrict__ dst, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        cs_st(dst, i, cs_ld(src, i));
}

__global__ void k_fill_i32(int32_t* p, int32_t v, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        p[i] = v;
}

// -------------------------------------------------------------------------------------
// host launchers
// -------------------------------------------------------------------------------------
int cs_tokens_launch(const cs_model* m, const int32_t* pending, const int32_t* draft,
                     const int32_t* draft_len, int B, int k, hipStream_t s) {
    k_tokens<<<B, 64, 0, s>>>(pending, draft, draft_len, k, m->cfg.vocab, m->tok);
    return cs_launch_ok("k_tokens");
}

int cs_rope_table_launch(const cs_model* m, const int32_t* kv_len, int B, int rows, hipStream_t s) {
    k_rope_table<<<B * rows, 64, 0, s>>>(kv_len, rows, m->cfg.head_dim / 2, m->cfg.head_dim,
                                         (double)m->cfg.rope_theta, m->rope_inv_freq, m->rope);
    return cs_launch_ok("k_rope_table");
}

int cs_embed_launch(const cs_model* m, const int32_t* tok, int R, hipStream_t s) {
    if (m->cfg.dtype == CS_BF16)
        k_embed<bf16_t><<<R, 256, 0, s>>>((const bf16_t*)m->embed, tok, m->cfg.d_model, m->x);
    else
        k_embed<float><<<R, 256, 0, s>>>((const float*)m->embed, tok, m->cfg.d_model, m->x);
    return cs_launch_ok("k_embed");
}

int cs_addnorm_launch(const cs_model* m, const float* part, int nparts,
                      const float* gain, void* xn_out, int R, int next_N, hipStream_t s) {
    const int d = m->cfg.d_model;
    const int64_t ps = (int64_t)R * d;
    if (xn_out && m->fast) {
        k_addnorm<f16_t><<<R, NORM_THREADS, 0, s>>>(m->x, part, nparts, ps, d, m->cfg.rms_eps, gain,
                                                    (f16_t*)xn_out, cs_gemm_x_tiled(R, next_N) ? 1 : 0,
                                                    m->range_flags);
    } else
        k_addnorm<float><<<R, NORM_THREADS, 0, s>>>(m->x, part, nparts, ps, d, m->cfg.rms_eps, gain,
                                                    (float*)xn_out, 0, nullptr);
    return cs_launch_ok("k_addnorm");
}

int cs_rope_append_launch(const cs_model* m, cs_kv* kv, int layer, const float* qkv, int nparts,
                          int rows, hipStream_t s) {
    const cs_model_cfg& c = m->cfg;
    const int R = kv->B * rows;
    const int64_t per_layer = (int64_t)kv->B * c.n_kv_heads * kv->cap * c.head_dim;
    const int64_t ps = (int64_t)R * (c.n_heads + 2 * c.n_kv_heads) * c.head_dim;
    const float2* rope = m->rope;
    const float* bias = m->layers[layer].bqkv;
    dim3 rgrid(c.n_heads + 2 * c.n_kv_heads, R);
    if (c.dtype == CS_BF16) {
        bf16_t* kc = (bf16_t*)kv->k + layer * per_layer;
        bf16_t* vc = (bf16_t*)kv->v + layer * per_layer;
        // many rows: the tiled version (needs 16-byte aligned quads: head_dim % 8 == 0)
        if (m->fast && R >= 4 * RA_ROWS && c.head_dim % 8 == 0 && c.head_dim <= 256) {
            dim3 grid(c.n_heads + 2 * c.n_kv_heads, (unsigned)cs_ceil_div(R, RA_ROWS));
            k_rope_append_rows<<<grid, RA_THREADS, 0, s>>>(qkv, nparts, ps, rope, kv->d_len, rows, R, c.n_heads,
                                                          c.n_kv_heads, c.head_dim, kv->cap, kc, vc,
                                                          (bf16_t*)m->q, bias);
        } else if (m->fast)
            k_rope_append<bf16_t, bf16_t><<<rgrid, 64, 0, s>>>(qkv, nparts, ps, rope, kv->d_len, rows,
                                                           c.n_heads, c.n_kv_heads, c.head_dim,
                                                           kv->cap, kc, vc, (bf16_t*)m->q, bias);
        else
            k_rope_append<bf16_t, float><<<rgrid, 64, 0, s>>>(qkv, nparts, ps, rope, kv->d_len, rows,
                                                          c.n_heads, c.n_kv_heads, c.head_dim,
                                                          kv->cap, kc, vc, (float*)m->q, bias);
    } else {
        float* kc = (float*)kv->k + layer * per_layer;
        float* vc = (float*)kv->v + layer * per_layer;
        k_rope_append<float, float><<<rgrid, 64, 0, s>>>(qkv, nparts, ps, rope, kv->d_len, rows,
                                                     c.n_heads, c.n_kv_heads, c.head_dim, kv->cap,
                                                     kc, vc, (float*)m->q, bias);
    }
    return cs_launch_ok("k_rope_append");
}

int cs_swiglu_launch(const cs_model* m, int R, hipStream_t s) {
    const int F = m->cfg.d_ff;
    dim3 grid((unsigned)cs_ceil_div(F, 256), R);
    k_swiglu<float><<<grid, 256, 0, s>>>(m->gu, F, (float*)m->act);   // plain path only
    return cs_launch_ok("k_swiglu");
}

int cs_argmax_accept_launch(const cs_model* m, const float* logits, int B, int k, int V,
                            const int32_t* draft, const int32_t* draft_len, int32_t* accepted,
                            int32_t* next_tok, int32_t* row_argmax_out, int32_t* kv_len,
                            int32_t* hist, int64_t hist_stride, int32_t* hist_len,
                            int32_t* room, hipStream_t s) {
    const int R = B * (k + 1);
    int nch = (int)cs_ceil_div(V, 8192);
    if (nch < 1) nch = 1;
    if (nch > m->am_chunks) nch = m->am_chunks;
    const int Vc = (int)cs_round_up(cs_ceil_div(V, nch), 4);
    nch = (int)cs_ceil_div(V, Vc);
    const int vec_ok = ((reinterpret_cast<uintptr_t>(logits) & 15) == 0) && (V % 4 == 0);
    dim3 grid(nch, R);
    const int pa = cs_prof_begin(CS_PROF_ARGMAX, s);
    k_argmax_partial<<<grid, AM_THREADS, 0, s>>>(logits, V, Vc, vec_ok, m->am_val_idx);
    cs_prof_end(pa, s);
    CS_TRY(cs_launch_ok("k_argmax_partial"));
    return cs_accept_launch(m, nch, B, k, draft, draft_len, accepted, next_tok, row_argmax_out, kv_len, hist,
                            hist_stride, hist_len, room, s);
}

int cs_accept_launch(const cs_model* m, int nch, int B, int k, const int32_t* draft,
                     const int32_t* draft_len, int32_t* accepted, int32_t* next_tok,
                     int32_t* row_argmax_out, int32_t* kv_len, int32_t* hist, int64_t hist_stride,
                     int32_t* hist_len, int32_t* room, hipStream_t s) {
    k_accept<<<B, ACC_THREADS, 0, s>>>(m->am_val_idx, nch, k, draft, draft_len, accepted, next_tok,
                                       m->row_argmax, row_argmax_out, kv_len, hist, hist_stride, hist_len,
                                       room);
    return cs_launch_ok("k_accept");
}

template <typename S>
static void convert_from(const S* src, void* dst, int dst_type, int64_t n, int blocks, hipStream_t s) {
    if (dst_type == CS_T_F32) k_convert<S, float><<<blocks, 256, 0, s>>>(src, (float*)dst, n);
    else if (dst_type == CS_T_BF16) k_convert<S, bf16_t><<<blocks, 256, 0, s>>>(src, (bf16_t*)dst, n);
    else k_convert<S, f16_t><<<blocks, 256, 0, s>>>(src, (f16_t*)dst, n);
}

int cs_convert_launch(const void* src, int src_type, void* dst, int dst_type, int64_t n,
                      hipStream_t s) {
    if (n <= 0) return CS_OK;
    const int blocks = (int)(cs_ceil_div(n, 256) < 4096 ? cs_ceil_div(n, 256) : 4096);
    if (src_type == CS_T_F32) convert_from((const float*)src, dst, dst_type, n, blocks, s);
    else if (src_type == CS_T_BF16) convert_from((const bf16_t*)src, dst, dst_type, n, blocks, s);
    else convert_from((const f16_t*)src, dst, dst_type, n, blocks, s);
    return cs_launch_ok("k_convert");
}

int cs_fill_i32_launch(int32_t* p, int32_t v, int64_t n, hipStream_t s) {
    if (n <= 0) return CS_OK;
    const int blocks = (int)(cs_ceil_div(n, 256) < 1024 ? cs_ceil_div(n, 256) : 1024);
    k_fill_i32<<<blocks, 256, 0, s>>>(p, v, n);
    return cs_launch_ok("k_fill_i32");
}
