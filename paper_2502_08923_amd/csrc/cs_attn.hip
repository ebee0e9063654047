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
// lane); V is cached transposed in 128-token blocks (token index contiguous) so its A operand is one 16-byte
// load per lane.  Softmax runs online in float32 (base 2), the row maximum is shared by the
// four lanes that hold a query row, and O is only rescaled when some maximum moved.
// The token range of a stream is split over workgroups, whose waves take its 32-token blocks in
// turn; a merge kernel combines the partial (max, sum, O) triples.
#include <type_traits>

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
        for (int t = part; t < cn; t += nparts) acc += sc[t] * cs_ld(V, cs_v_index(c0 + t, d, hd));
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
// max over the four lanes {c, c+16, c+32, c+48} that share a query row, with the row-swap
// instructions of gfx950 (two register swaps and two max) instead of two round trips through
// the LDS crossbar: swapping x with itself leaves (low half, low half) and (high half, high
// half) in the two results, whose max is the reduction over lanes 32 apart; then 16 apart.
__device__ __forceinline__ float fa_row4_max(float x) {
    const unsigned u = __float_as_uint(x);
    const auto r32 = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const float m = fmaxf(__uint_as_float(r32[0]), __uint_as_float(r32[1]));
    const unsigned v = __float_as_uint(m);
    const auto r16 = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return fmaxf(__uint_as_float(r16[0]), __uint_as_float(r16[1]));
}

#define FA_QROWS (16 * FA_NT)
#define FA_RESCALE_LOG2 8.0f
#define FA_OPAD 4          // LDS row padding (floats) of the in-workgroup merge buffers

// attention output element: float16 outputs feed the output projection and are saturated
__device__ __forceinline__ void fa_store_out(f16_t* p, int64_t i, float v, bool& hit) { p[i] = cs_f16_sat(v, hit); }
__device__ __forceinline__ void fa_store_out(float* p, int64_t i, float v, bool&) { p[i] = v; }

template <int HD>
struct fa_kbuf { bf16x8 k[2][HD / 32]; };
template <int HD>
struct fa_vbuf { bf16x8 v[HD / 16]; };

// Partial layout: po[item][split][qrow][HD] float, pml[item][split][qrow][2] = (max2, sum)
// where item = (b*KVH + kvh)*nqg + qg, split = workgroup index along the token axis and max2
// is the reference maximum in base-2 scaled units.  A split whose token range is empty
// writes (max2 = -inf, 0, 0).
// With `fr.qkv` set the kernel also does what k_rope_append does, for what it needs itself:
// the query tile is built from the split-K partial tiles of the q/k/v projection (summed in the
// same order, rotated, rounded), and the workgroup that owns the token range of a new row
// writes that row's K and V into the cache before anybody in the workgroup reads it.  Nobody
// else needs the row in this launch: a workgroup only reads cache rows of its own ranges.
struct fa_fused_rope {
    const float* qkv;        // [nparts][R][(H + 2*KVH) * HD] partial tiles, or NULL: q is given
    int nparts;
    int64_t part_stride;
    const float2* rope;      // [R][HD/2] (cos, sin)
    bf16_t* kc_w;            // this layer's caches, writable
    bf16_t* vc_w;
    const float* bias;       // [(H + 2*KVH) * HD] biases of the q, k, v projections, or NULL
};

template <int HD>
__global__ __launch_bounds__(256) void k_attn_mfma(const bf16_t* __restrict__ q,
                                                   const bf16_t* __restrict__ kc,
                                                   const bf16_t* __restrict__ vc,
                                                   const int32_t* __restrict__ kv_len, int rows,
                                                   int H, int KVH, int64_t cap, int Tw, int nqg,
                                                   int nsplit, float* __restrict__ po,
                                                   float* __restrict__ pml, fa_fused_rope fr) {
    constexpr int KS = HD / 32;      // MFMA k-steps over the head dimension
    constexpr int MT = HD / 16;      // 16-row tiles of O^T
    constexpr int OROW = HD + FA_OPAD;
    constexpr int QROW = HD * 2 + 16;                 // bytes per query row in LDS (padded)
    constexpr int MERGE_BYTES = 2 * FA_QROWS * OROW * 4 + 2 * FA_QROWS * 2 * 4;
    constexpr int Q_BYTES = FA_QROWS * QROW;
    // the query tile (read during the main loop) and the merge buffers (used after it)
    // share the same LDS
    __shared__ __attribute__((aligned(16))) unsigned char smem[MERGE_BYTES > Q_BYTES ? MERGE_BYTES : Q_BYTES];
    float* s_o = reinterpret_cast<float*>(smem);                          // [2][FA_QROWS*OROW]
    float* s_ml = reinterpret_cast<float*>(smem) + 2 * FA_QROWS * OROW;   // [2][FA_QROWS*2]
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int qg = blockIdx.x % nqg;
    const int split = blockIdx.x / nqg;
    const int wg = split * 4 + wave;                    // wave index along the token axis
    const int kvh = blockIdx.y, b = blockIdx.z;
    const int G = H / KVH;
    const int QR = G * rows;
    const int L = kv_len[b];
    const int n_tok = L + rows;
    // The workgroup's token range is 4*Tw long; its four waves take the 32-token blocks of it in
    // turn (wave w: blocks w, w+4, ...), so that at any time the workgroup reads neighbouring
    // blocks: the four 64-byte pieces a V row contributes then form one 256-byte run.
    constexpr int STEP = 4 * 32;
    const int w_begin = min(split * 4 * Tw, n_tok);
    const int t_end = min(n_tok, w_begin + 4 * Tw);
    const int t_begin = w_begin + 32 * wave;            // may lie past t_end: no blocks then
    // blocks that lie completely inside the old cache need neither mask nor clean-up
    const int t_split = max(w_begin, min(t_end, (L / 32) * 32));
    // first block of this wave at or beyond t_split
    const int t_tail = t_begin >= t_split ? t_begin : t_begin + (t_split - t_begin + STEP - 1) / STEP * STEP;
    (void)wg;
    const bf16_t* __restrict__ K = kc + ((int64_t)b * KVH + kvh) * cap * HD;
    const bf16_t* __restrict__ V = vc + ((int64_t)b * KVH + kvh) * HD * cap;

    // stage the query tile: global qrow n = qg*48 + local row  <->  block row n / G, head n % G
    if (fr.qkv == nullptr) {
        for (int idx = tid; idx < FA_QROWS * (HD / 8); idx += 256) {
            const int row = idx / (HD / 8), seg = idx % (HD / 8);
            const int n = qg * FA_QROWS + row;
            bf16x8 v = (bf16x8){0, 0, 0, 0, 0, 0, 0, 0};
            if (n < QR) {
                const int i = n / G, gq = n % G;
                v = *reinterpret_cast<const bf16x8*>(
                    q + (((int64_t)(b * rows + i)) * H + kvh * G + gq) * HD + seg * 8);
            }
            *reinterpret_cast<bf16x8*>(smem + row * QROW + seg * 16) = v;
        }
    } else {
        constexpr int HALF = HD / 2, SEGS = HALF / 8;        // 8-element segments per half head
        const int nqkv = (H + 2 * KVH) * HD;
        // elements j0..j0+7 and HALF+j0..HALF+j0+7 of one head of block row r: partial tiles
        // summed in order, the pair (j, HALF + j) rotated by the row's angle j
        auto head_pair = [&](int r, int head, int j0, bool rotate, bf16x8& lo, bf16x8& hi) {
            const float* __restrict__ src = fr.qkv + (int64_t)r * nqkv + (int64_t)head * HD + j0;
            float a[8], cc[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) a[u] = cc[u] = 0.f;
            for (int p = 0; p < fr.nparts; ++p) {
                const float* __restrict__ sp = src + p * fr.part_stride;
                const f32x4 a0 = *reinterpret_cast<const f32x4*>(sp), a1 = *reinterpret_cast<const f32x4*>(sp + 4);
                const f32x4 c0 = *reinterpret_cast<const f32x4*>(sp + HALF), c1 = *reinterpret_cast<const f32x4*>(sp + HALF + 4);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    a[u] += a0[u];
                    a[4 + u] += a1[u];
                    cc[u] += c0[u];
                    cc[4 + u] += c1[u];
                }
            }
            if (fr.bias) {                            // projection bias, before the rotation
                const float* __restrict__ bp = fr.bias + head * HD + j0;
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    a[u] += bp[u];
                    cc[u] += bp[HALF + u];
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                float x = a[u], y = cc[u];
                if (rotate) {
                    const float2 cs = fr.rope[(int64_t)r * HALF + j0 + u];
                    const float rx = x * cs.x - y * cs.y;
                    const float ry = y * cs.x + x * cs.y;
                    x = rx;
                    y = ry;
                }
                lo[u] = (bf16_t)x;
                hi[u] = (bf16_t)y;
            }
        };
        // first the new rows whose position lies in this workgroup's token range (4*Tw long):
        // their stores complete while the query tile is being built
        bf16_t* Kw = fr.kc_w + ((int64_t)b * KVH + kvh) * cap * HD;
        bf16_t* Vw = fr.vc_w + ((int64_t)b * KVH + kvh) * HD * cap;
        if (qg == 0) {
            for (int idx = tid; idx < rows * SEGS; idx += 256) {
                const int i = idx / SEGS, sg = idx % SEGS;
                const int pos = L + i;
                if ((pos / Tw) >> 2 != split) continue;
                bf16x8 lo, hi;
                head_pair(b * rows + i, H + kvh, sg * 8, true, lo, hi);
                *reinterpret_cast<bf16x8*>(Kw + (int64_t)pos * HD + sg * 8) = lo;
                *reinterpret_cast<bf16x8*>(Kw + (int64_t)pos * HD + HALF + sg * 8) = hi;
                head_pair(b * rows + i, H + KVH + kvh, sg * 8, false, lo, hi);
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    Vw[cs_v_index(pos, sg * 8 + u, HD)] = lo[u];
                    Vw[cs_v_index(pos, HALF + sg * 8 + u, HD)] = hi[u];
                }
            }
        }
        for (int idx = tid; idx < FA_QROWS * SEGS; idx += 256) {
            const int row = idx / SEGS, sg = idx % SEGS;
            const int n = qg * FA_QROWS + row;
            bf16x8 lo = (bf16x8){0, 0, 0, 0, 0, 0, 0, 0}, hi = lo;
            if (n < QR) head_pair(b * rows + n / G, kvh * G + n % G, sg * 8, true, lo, hi);
            *reinterpret_cast<bf16x8*>(smem + row * QROW + sg * 16) = lo;
            *reinterpret_cast<bf16x8*>(smem + row * QROW + HD + sg * 16) = hi;
        }
    }
    int qi[FA_NT];               // block row index of the lane's query row (for the causal mask)
#pragma unroll
    for (int nt = 0; nt < FA_NT; ++nt) {
        const int n = qg * FA_QROWS + nt * 16 + c;
        qi[nt] = n < QR ? n / G : -1;
    }
    __syncthreads();

    f32x4 oacc[MT][FA_NT], lacc[FA_NT];
#pragma unroll
    for (int nt = 0; nt < FA_NT; ++nt) {
        lacc[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) oacc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    float m_run[FA_NT];
#pragma unroll
    for (int nt = 0; nt < FA_NT; ++nt) m_run[nt] = -INFINITY;

    const float scale2 = 1.4426950408889634f / sqrtf((float)HD);
    const bf16_t one = (bf16_t)1.0f;
    const bf16x8 ones = (bf16x8){one, one, one, one, one, one, one, one};

    // K tile a, MFMA row m=c  <->  token t0 + 8*(c/4) + 4a + c%4
    const int ktok0 = 8 * (c >> 2) + (c & 3);
    auto load_k_from = [&](const bf16_t* Kb, fa_kbuf<HD>& buf, int t0, int limit) {
        if (t0 >= limit) return;
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            // the four lanes of a token row read 64 contiguous bytes per k-step
            const bf16_t* kp = Kb + (int64_t)(t0 + ktok0 + 4 * a) * HD + g * 8;
#pragma unroll
            for (int s = 0; s < KS; ++s) buf.k[a][s] = *reinterpret_cast<const bf16x8*>(kp + s * 32);
        }
    };
    auto load_v_from = [&](const bf16_t* Vb, fa_vbuf<HD>& buf, int t0, int limit) {
        if (t0 >= limit) return;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            buf.v[mt] = *reinterpret_cast<const bf16x8*>(Vb + cs_v_index(t0 + 8 * g, mt * 16 + c, HD));
    };
    auto load_k = [&](fa_kbuf<HD>& buf, int t0, int limit) { load_k_from(K, buf, t0, limit); };
    auto load_v = [&](fa_vbuf<HD>& buf, int t0, int limit) { load_v_from(V, buf, t0, limit); };

    auto compute = [&](fa_kbuf<HD>& kb, fa_vbuf<HD>& vb, int t0, auto tail_tag) {
        constexpr bool TAIL = decltype(tail_tag)::value;
        // scores: lane (c, g) gets tokens t0 + 8g + (4a + j) of query row nt*16 + c
        f32x4 sacc[2][FA_NT];
#pragma unroll
        for (int nt = 0; nt < FA_NT; ++nt) {
            f32x4 z0 = (f32x4){0.f, 0.f, 0.f, 0.f}, z1 = z0;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const bf16x8 qb = *reinterpret_cast<const bf16x8*>(
                    smem + (nt * 16 + c) * QROW + s * 64 + g * 16);
                z0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb.k[0][s], qb, z0, 0, 0, 0);
                z1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb.k[1][s], qb, z1, 0, 0, 0);
            }
            sacc[0][nt] = z0;
            sacc[1][nt] = z1;
        }
        if (TAIL) {
            // dead cache rows may hold anything: zero their V so that 0 * garbage stays 0
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (t0 + 8 * g + j >= n_tok) vb.v[mt][j] = (bf16_t)0.f;
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
                    float s = sacc[a][nt][j];
                    if (TAIL && (t0 + 8 * g + 4 * a + j > L + qi[nt])) s = -INFINITY;
                    sv[4 * a + j] = s;
                }
            float mx = fmaxf(fmaxf(sv[0], sv[1]), sv[2]);
            mx = fmaxf(fmaxf(mx, sv[3]), sv[4]);
            mx = fmaxf(fmaxf(mx, sv[5]), fmaxf(sv[6], sv[7]));
            mx = fa_row4_max(mx);                                  // over the lanes c, c+16, c+32, c+48
            mx *= scale2;                       // scale2 > 0: scaling commutes with the max
            // The reference maximum only follows the true one when it is left behind by more
            // than 2^8: probabilities stay below 256, O and the row sum stay consistent, and
            // the rescale of O (the expensive part) runs a handful of times per wave.
            const bool up = mx > m_run[nt] + FA_RESCALE_LOG2;
            const float m_new = up ? mx : m_run[nt];
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
            alpha[nt] = up ? __builtin_amdgcn_exp2f(m_run[nt] - m_safe) : 1.0f;
            moved |= up;
            m_run[nt] = m_new;
#pragma unroll
            for (int j = 0; j < 8; ++j)
                pb[nt][j] = (bf16_t)__builtin_amdgcn_exp2f(fmaf(sv[j], scale2, -m_safe));
        }
        if (__any(moved)) {
            // rare path (see above); the empty asm statements keep the register-file copies
            // that the multiply needs inside this branch
#pragma unroll
            for (int nt = 0; nt < FA_NT; ++nt) {
                asm volatile("" : "+a"(lacc[nt]));
                lacc[nt] *= alpha[nt];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    asm volatile("" : "+a"(oacc[mt][nt]));
                    oacc[mt][nt] *= alpha[nt];
                }
            }
        }
#pragma unroll
        for (int nt = 0; nt < FA_NT; ++nt) {
            // row sums of the rounded probabilities on the matrix core: ones^T * P^T
            lacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[nt], lacc[nt], 0, 0, 0);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                oacc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vb.v[mt], pb[nt], oacc[mt][nt], 0, 0, 0);
        }
        // keep the accumulators in the accumulation registers between blocks, so that the
        // vector registers stay free for the K/V stages (no register-file shuffling per block)
#pragma unroll
        for (int nt = 0; nt < FA_NT; ++nt) {
            asm volatile("" : "+a"(lacc[nt]));
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) asm volatile("" : "+a"(oacc[mt][nt]));
        }
    };
    const std::integral_constant<bool, false> main_tag;
    const std::integral_constant<bool, true> tail_tag;

    // register stages: K is fetched two 32-token blocks ahead, V one block ahead, so about
    // 24 KB per wave are in flight while one block is being multiplied
    {
        fa_kbuf<HD> k0, k1, k2;
        fa_vbuf<HD> v0, v1;
        // this wave's unmasked blocks are t_begin + j*STEP, j < n.  Every workgroup starts at a
        // different j (and wraps): the workgroups of a launch run in step, and with all of them at
        // the same relative position some cache pitches put them on the same memory channels
        const int e = t_split;
        const int n = t_begin < e ? (e - t_begin + STEP - 1) / STEP : 0;
        const int wg_id = (b * KVH + kvh) * nsplit + split;
        const int n_wg = w_begin < e ? (e - w_begin + STEP - 1) / STEP : 0;       // wave 0's count
        const int rot_wg = n_wg > 0 ? (int)(((int64_t)wg_id * 2654435761LL >> 8) % n_wg) : 0;
        const int rot = n > 0 ? min(rot_wg, n - 1) : 0;     // the same round for all four waves
        auto at = [&](int i) {
            int j = i + rot;
            j = j >= n ? j - n : j;
            return t_begin + j * STEP;
        };
        auto ldk = [&](fa_kbuf<HD>& buf, int i) { if (i < n) load_k(buf, at(i), e); };
        auto ldv = [&](fa_vbuf<HD>& buf, int i) { if (i < n) load_v(buf, at(i), e); };
        ldk(k0, 0);
        ldv(v0, 0);
        ldk(k1, 1);
        for (int i = 0; i < n; i += 6) {
            ldv(v1, i + 1);  ldk(k2, i + 2);  compute(k0, v0, 0, main_tag);
            if (i + 1 >= n) break;
            ldv(v0, i + 2);  ldk(k0, i + 3);  compute(k1, v1, 0, main_tag);
            if (i + 2 >= n) break;
            ldv(v1, i + 3);  ldk(k1, i + 4);  compute(k2, v0, 0, main_tag);
            if (i + 3 >= n) break;
            ldv(v0, i + 4);  ldk(k2, i + 5);  compute(k0, v1, 0, main_tag);
            if (i + 4 >= n) break;
            ldv(v1, i + 5);  ldk(k0, i + 6);  compute(k1, v0, 0, main_tag);
            if (i + 5 >= n) break;
            ldv(v0, i + 6);  ldk(k1, i + 7);  compute(k2, v1, 0, main_tag);
        }
    }
    // the few blocks that touch the new rows or the dead region: masked, not pipelined
    // With the fused append the rows at and beyond L were written by this workgroup, above, through
    // the writable cache pointers; K and V promise the compiler memory that nobody writes, so these
    // blocks are read through pointers derived from the writable ones (after the barrier above).
    const bf16_t* K_tail = fr.qkv ? fr.kc_w + ((int64_t)b * KVH + kvh) * cap * HD : K;
    const bf16_t* V_tail = fr.qkv ? fr.vc_w + ((int64_t)b * KVH + kvh) * HD * cap : V;
    for (int t0 = t_tail; t0 < t_end; t0 += STEP) {
        fa_kbuf<HD> kt;
        fa_vbuf<HD> vt;
        load_k_from(K_tail, kt, t0, t_end);
        load_v_from(V_tail, vt, t0, t_end);
        compute(kt, vt, t0, tail_tag);
    }
    __syncthreads();             // every wave is done with the query tile: LDS changes hands

    float l_tot[FA_NT];
#pragma unroll
    for (int nt = 0; nt < FA_NT; ++nt) l_tot[nt] = lacc[nt][0];

    // merge the four waves through LDS: (2,3) -> (0,1), then 1 -> 0
    auto put = [&](int slot) {
        float* so = s_o + slot * FA_QROWS * OROW;
        float* sm = s_ml + slot * FA_QROWS * 2;
#pragma unroll
        for (int nt = 0; nt < FA_NT; ++nt) {
            const int n = nt * 16 + c;
            if (g == 0) { sm[n * 2] = m_run[nt]; sm[n * 2 + 1] = l_tot[nt]; }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                *reinterpret_cast<f32x4*>(&so[n * OROW + mt * 16 + 4 * g]) = oacc[mt][nt];
        }
    };
    auto take = [&](int slot) {
        const float* so = s_o + slot * FA_QROWS * OROW;
        const float* sm = s_ml + slot * FA_QROWS * 2;
#pragma unroll
        for (int nt = 0; nt < FA_NT; ++nt) {
            const int n = nt * 16 + c;
            const float mb = sm[n * 2], lb = sm[n * 2 + 1];
            const float M = fmaxf(m_run[nt], mb);
            const float Ms = (M == -INFINITY) ? 0.f : M;
            const float sa = __builtin_amdgcn_exp2f(m_run[nt] - Ms);
            const float sb = __builtin_amdgcn_exp2f(mb - Ms);
            m_run[nt] = M;
            l_tot[nt] = l_tot[nt] * sa + lb * sb;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const f32x4 ob = *reinterpret_cast<const f32x4*>(&so[n * OROW + mt * 16 + 4 * g]);
                oacc[mt][nt] = oacc[mt][nt] * sa + ob * sb;
            }
        }
    };
    if (wave >= 2) put(wave - 2);
    __syncthreads();
    if (wave < 2) take(wave);
    __syncthreads();
    if (wave == 1) put(0);
    __syncthreads();
    if (wave != 0) return;
    take(0);

    const int64_t item = ((int64_t)b * KVH + kvh) * nqg + qg;
    float* __restrict__ o_out = po + (item * nsplit + split) * FA_QROWS * HD;
    float* __restrict__ ml_out = pml + (item * nsplit + split) * FA_QROWS * 2;
#pragma unroll
    for (int nt = 0; nt < FA_NT; ++nt) {
        const int n = nt * 16 + c;
        if (g == 0) { ml_out[n * 2] = m_run[nt]; ml_out[n * 2 + 1] = l_tot[nt]; }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            *reinterpret_cast<f32x4*>(o_out + (int64_t)n * HD + mt * 16 + 4 * g) = oacc[mt][nt];
    }
}

// -------------------------------------------------------------------------------------
// tuned kernel for wide blocks (more than 48 query rows per KV head, e.g. k = 32: 132 rows)
//
// Up to FA_QG consumer waves each own one 48-row query group and all walk the same token
// range; one producer wave streams K and V from HBM once per workgroup and lays them into a
// three-stage LDS ring in MFMA fragment order, so the KV bytes are read once however many
// query groups share them.  One barrier per 32-token block hands the stages over.  Every
// consumer writes its own partial (no in-workgroup merge); k_attn_merge combines the splits.
// -------------------------------------------------------------------------------------
#define FA_QG 3
#define FA_STAGES 3
#define FA_TEAMS 2          // (FA_QG consumers + 1 producer) per team; two waves per SIMD
#define FA_LDS_THREADS (64 * (FA_QG + 1) * FA_TEAMS)

template <int HD>
__global__ __launch_bounds__(FA_LDS_THREADS) void k_attn_lds(const bf16_t* __restrict__ q,
                                                              const bf16_t* __restrict__ kc,
                                                              const bf16_t* __restrict__ vc,
                                                              const int32_t* __restrict__ kv_len,
                                                              int rows, int H, int KVH, int64_t cap,
                                                              int Tw, int nqg, int nqgw, int nsplit,
                                                              int ranges, float* __restrict__ po,
                                                              float* __restrict__ pml) {
    constexpr int KS = HD / 32, MT = HD / 16;
    constexpr int QROW = HD * 2 + 16;
    constexpr int K_BYTES = 2 * KS * 1024, V_BYTES = MT * 1024;
    constexpr int STAGE_BYTES = K_BYTES + V_BYTES;
    __shared__ __attribute__((aligned(16))) unsigned char stage_all[FA_TEAMS][FA_STAGES][STAGE_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char qs[FA_QG][FA_QROWS * QROW];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int c = lane & 15, g = lane >> 4;
    // Workgroup -> (stream, KV head, token range pair, group of query groups).  The nqgw
    // workgroups that walk the same K/V range (long blocks, e.g. prompt ingestion) get ids 8
    // apart: consecutive ids go to different XCDs, each with its own L2, so this puts them on
    // one XCD at about the same time and the range is fetched from HBM once, not nqgw times.
    const int nsp = nsplit / FA_TEAMS;                  // ranges = B * KVH * nsp
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int range = (slot / nqgw) * 8 + xcd;
    if (range >= ranges) return;                        // whole workgroup, before any barrier
    // which group of FA_QG query groups: the last rows of a block see the most tokens (see n_lim
    // below), so they are dispatched first and the short ones fill the tail of the launch
    const int qgw = nqgw - 1 - slot % nqgw;
    // Roles of the eight waves (hardware waves go to the four SIMDs in turn: wave w runs on SIMD
    // w % 4).  With three live query groups per team: waves 0-2 and 4-6 are the consumers of teams 0
    // and 1, waves 3 and 7 the producers, so every consumer SIMD carries one consumer of each team.
    // With at most two live groups (e.g. 11 block rows of seven or eight query heads per KV head)
    // the four live consumers get a SIMD each: waves 0-3 = (team 0, group 0), (0, 1), (1, 0), (1, 1),
    // waves 4 and 5 the producers, waves 6 and 7 the dead third groups.
    const int hw = tid >> 6;
    const int live_groups = min(FA_QG, nqg - qgw * FA_QG);
    const bool spread = live_groups <= 2;
    const int team = spread ? (hw < 4 ? hw >> 1 : (hw & 1)) : hw / (FA_QG + 1);
    const int wave = spread ? (hw < 4 ? (hw & 1) : (hw < 6 ? FA_QG : 2)) : hw % (FA_QG + 1);
    unsigned char (*stage)[STAGE_BYTES] = stage_all[team];
    const int split = (range % nsp) * FA_TEAMS + team;  // number of this team's partial result
    const int kvh = (range / nsp) % KVH, b = range / (nsp * KVH);
    const int G = H / KVH;
    const int QR = G * rows;
    const int L = kv_len[b];
    const int n_tok = L + rows;
    // Causality: block row i sees the tokens up to L + i, so nothing beyond the last row of this
    // workgroup's query groups is walked (long prompt blocks: the upper triangle of the block).
    const int last_row = min(rows - 1, ((qgw + 1) * FA_QG * FA_QROWS - 1) / G);
    const int n_lim = L + last_row + 1;
    // The two teams share the workgroup's token range of FA_TEAMS*Tw and take its 32-token blocks
    // in turn (team t: blocks t, t+2, ...), so the workgroup reads neighbouring blocks together.
    // `split` still numbers the partial result: (range, team).
    constexpr int TSTEP = 32 * FA_TEAMS;
    const int w_begin = min((split - team) * Tw, n_lim);
    const int w_blocks = (min(n_lim, w_begin + FA_TEAMS * Tw) - w_begin + 31) / 32;
    const int t_begin = w_begin + 32 * team;
    const int nblocks = (w_blocks - team + FA_TEAMS - 1) / FA_TEAMS;
    // both teams pass the same number of barriers: team 0's count
    const int nblocks_wg = (w_blocks + FA_TEAMS - 1) / FA_TEAMS;
    const bf16_t* __restrict__ K = kc + ((int64_t)b * KVH + kvh) * cap * HD;
    const bf16_t* __restrict__ V = vc + ((int64_t)b * KVH + kvh) * HD * cap;

    // stage the query tiles of all groups of this workgroup
    for (int idx = tid; idx < FA_QG * FA_QROWS * (HD / 8); idx += FA_LDS_THREADS) {
        const int grp = idx / (FA_QROWS * (HD / 8));
        const int rem = idx % (FA_QROWS * (HD / 8));
        const int row = rem / (HD / 8), seg = rem % (HD / 8);
        const int n = (qgw * FA_QG + grp) * FA_QROWS + row;
        bf16x8 v = (bf16x8){0, 0, 0, 0, 0, 0, 0, 0};
        if (n < QR) {
            const int i = n / G, gq = n % G;
            v = *reinterpret_cast<const bf16x8*>(
                q + (((int64_t)(b * rows + i)) * H + kvh * G + gq) * HD + seg * 8);
        }
        *reinterpret_cast<bf16x8*>(&qs[grp][row * QROW + seg * 16]) = v;
    }

    const int ktok0 = 8 * (c >> 2) + (c & 3);
    if (wave == FA_QG) {
        // ---------------- producer: K/V blocks -> LDS ring ----------------
        bf16x8 kr[3][2][KS], vr[3][MT];       // three blocks in flight in registers (block j in slot j % 3)
        auto load = [&](int slot, int blk) {
            const int bl = blk < nblocks ? blk : (nblocks > 0 ? nblocks - 1 : 0);   // clamped
            const int t0 = (nblocks > 0 ? t_begin : 0) + bl * TSTEP;
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                const bf16_t* kp = K + (int64_t)(t0 + ktok0 + 4 * a) * HD + g * 8;
#pragma unroll
                for (int s = 0; s < KS; ++s)
                    kr[slot][a][s] = *reinterpret_cast<const bf16x8*>(kp + s * 32);
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                vr[slot][mt] = *reinterpret_cast<const bf16x8*>(V + cs_v_index(t0 + 8 * g, mt * 16 + c, HD));
        };
        auto store = [&](int slot, int st, int blk) {
            const int t0 = (nblocks > 0 ? t_begin : 0) + (blk < nblocks ? blk : (nblocks > 0 ? nblocks - 1 : 0)) * TSTEP;
            unsigned char* sp = stage[st];
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int s = 0; s < KS; ++s)
                    *reinterpret_cast<bf16x8*>(sp + ((a * KS + s) * 64 + lane) * 16) = kr[slot][a][s];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                bf16x8 v = vr[slot][mt];
                // dead cache rows may hold anything: zero their V so that 0 * garbage stays 0
                if (t0 + 32 > n_tok) {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (t0 + 8 * g + j >= n_tok) v[j] = (bf16_t)0.f;
                }
                *reinterpret_cast<bf16x8*>(sp + K_BYTES + (mt * 64 + lane) * 16) = v;
            }
        };
        // an empty range still loads (clamped to block 0 of the cache, always allocated) and
        // stores into stages nobody reads; the barrier count is the workgroup's, not the team's
        load(0, 0);
        load(1, 1);
        load(2, 2);
        store(0, 0, 0);
        load(0, 3);
        store(1, 1, 1);
        load(1, 4);
        __syncthreads();                                   // stages 0, 1 and the query tiles are ready
        static_assert(FA_STAGES == 3, "block j: register slot j % 3, LDS stage j % 3");
        for (int i = 0; i < nblocks_wg; i += 3) {
            // consumer iteration i reads stages i and i+1: block i+2 goes to stage (i+2)%3, which
            // held block i-1; its register slot is refilled with block i+5, so blocks i+3, i+4
            // and i+5 (48 KB) are in flight while block i is being multiplied
            store(2, 2, i + 2);
            load(2, i + 5);
            __syncthreads();
            if (i + 1 >= nblocks_wg) break;
            store(0, 0, i + 3);
            load(0, i + 6);
            __syncthreads();
            if (i + 2 >= nblocks_wg) break;
            store(1, 1, i + 4);
            load(1, i + 7);
            __syncthreads();
        }
        return;
    }

    // ---------------- consumers: one 48-row query group each ----------------
    const int qg = qgw * FA_QG + wave;
    const bool live = qg < nqg;
    const unsigned char* myq = qs[wave];
    int qi[FA_NT];
#pragma unroll
    for (int nt = 0; nt < FA_NT; ++nt) {
        const int n = qg * FA_QROWS + nt * 16 + c;
        qi[nt] = n < QR ? n / G : -1;
    }
    f32x4 oacc[MT][FA_NT], lacc[FA_NT];
#pragma unroll
    for (int nt = 0; nt < FA_NT; ++nt) {
        lacc[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) oacc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    float m_run[FA_NT], thr[FA_NT];
#pragma unroll
    for (int nt = 0; nt < FA_NT; ++nt) m_run[nt] = thr[nt] = -INFINITY;
    const float scale2 = 1.4426950408889634f / sqrtf((float)HD);
    const float inv_scale2 = sqrtf((float)HD) / 1.4426950408889634f;
    const bf16_t one = (bf16_t)1.0f;
    const bf16x8 ones = (bf16x8){one, one, one, one, one, one, one, one};

    // scores of one block: S^T = K Q^T from the K fragments of stage `sp`
    // the wave's query fragments stay in registers for the whole token range (read once from
    // the staged tile, after the first barrier below)
    constexpr int QS_REG = KS;          // k-steps whose query fragments stay in registers (all of them fit)
    bf16x8 qreg[FA_NT][QS_REG];
    auto q_lds = [&](int nt, int s) {
        return *reinterpret_cast<const bf16x8*>(myq + (nt * 16 + c) * QROW + s * 64 + g * 16);
    };
    auto load_q = [&]() {
#pragma unroll
        for (int nt = 0; nt < FA_NT; ++nt)
#pragma unroll
            for (int s = 0; s < QS_REG; ++s) qreg[nt][s] = q_lds(nt, s);
    };
    auto scores = [&](const unsigned char* sp, f32x4 (&sacc)[2][FA_NT]) {
        // all K fragments of the block are requested at once (LDS latency is ~100 cycles and
        // only two waves share a SIMD, so fragments are read well ahead of their use)
        bf16x8 kf[2][KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            kf[0][s] = *reinterpret_cast<const bf16x8*>(sp + ((0 * KS + s) * 64 + lane) * 16);
            kf[1][s] = *reinterpret_cast<const bf16x8*>(sp + ((1 * KS + s) * 64 + lane) * 16);
        }
#pragma unroll
        for (int nt = 0; nt < FA_NT; ++nt) {
            f32x4 z0 = (f32x4){0.f, 0.f, 0.f, 0.f}, z1 = z0;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const bf16x8 qf = s < QS_REG ? qreg[nt][s] : q_lds(nt, s);
                z0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][s], qf, z0, 0, 0, 0);
                z1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[1][s], qf, z1, 0, 0, 0);
            }
            sacc[0][nt] = z0;
            sacc[1][nt] = z1;
        }
    };
    // ---- the pieces of one block's softmax and PV ----
    auto score_of = [&](const f32x4 (&sacc)[2][FA_NT], int nt, int e, int t0, auto tail_tag) {   // e = 4a + j
        constexpr bool TAIL = decltype(tail_tag)::value;
        const float sc = sacc[e >> 2][nt][e & 3];
        return (TAIL && (t0 + 8 * g + e > L + qi[nt])) ? -INFINITY : sc;
    };
    // reference maxima: leaves m_run (and O, rescaled if a reference moved) ready for `prob`
    auto reference = [&](const f32x4 (&sacc)[2][FA_NT], int t0, auto tail_tag) {
        constexpr bool TAIL = decltype(tail_tag)::value;
        // Common case first: no score of the block is more than 2^8 above its row's reference
        // maximum.  Then the reference stays, nothing is rescaled, and the exact row maximum
        // (a reduction across the four lanes that share a row) is not needed at all: every lane
        // only compares its own eight scores with the row's threshold.
        bool calm = false;
        if (!TAIL) {
            bool over = false;
#pragma unroll
            for (int nt = 0; nt < FA_NT; ++nt) {
                const float lm = fmaxf(fmaxf(fmaxf(sacc[0][nt][0], sacc[0][nt][1]), fmaxf(sacc[0][nt][2], sacc[0][nt][3])),
                                       fmaxf(fmaxf(sacc[1][nt][0], sacc[1][nt][1]), fmaxf(sacc[1][nt][2], sacc[1][nt][3])));
                over |= !(lm <= thr[nt]);          // also true while the reference is still -inf
            }
            calm = !__any(over);
        }
        if (calm) return;
        bool moved = false;
        float alpha[FA_NT];
#pragma unroll
        for (int nt = 0; nt < FA_NT; ++nt) {
            float mx = fmaxf(fmaxf(score_of(sacc, nt, 0, t0, tail_tag), score_of(sacc, nt, 1, t0, tail_tag)),
                             score_of(sacc, nt, 2, t0, tail_tag));
            mx = fmaxf(fmaxf(mx, score_of(sacc, nt, 3, t0, tail_tag)), score_of(sacc, nt, 4, t0, tail_tag));
            mx = fmaxf(fmaxf(mx, score_of(sacc, nt, 5, t0, tail_tag)),
                       fmaxf(score_of(sacc, nt, 6, t0, tail_tag), score_of(sacc, nt, 7, t0, tail_tag)));
            mx = fa_row4_max(mx);                              // over the lanes c, c+16, c+32, c+48
            mx *= scale2;
            const bool up = mx > m_run[nt] + FA_RESCALE_LOG2;  // see k_attn_mfma
            const float m_new = up ? mx : m_run[nt];
            alpha[nt] = up ? __builtin_amdgcn_exp2f(m_run[nt] - ((m_new == -INFINITY) ? 0.f : m_new)) : 1.0f;
            moved |= up;
            m_run[nt] = m_new;
            // scores above this leave the calm path (raw score units; -inf while no score has
            // been seen, so that the comparison above fails)
            thr[nt] = (m_new == -INFINITY) ? -INFINITY : (m_new + FA_RESCALE_LOG2) * inv_scale2;
        }
        if (__any(moved)) {
#pragma unroll
            for (int nt = 0; nt < FA_NT; ++nt) {
                lacc[nt] *= alpha[nt];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) oacc[mt][nt] *= alpha[nt];
            }
        }
    };
    auto prob = [&](const f32x4 (&sacc)[2][FA_NT], int nt, int e, int t0, auto tail_tag) {
        const float m_safe = (m_run[nt] == -INFINITY) ? 0.f : m_run[nt];
        return (bf16_t)__builtin_amdgcn_exp2f(fmaf(score_of(sacc, nt, e, t0, tail_tag), scale2, -m_safe));
    };
    auto pv = [&](const unsigned char* sp, const bf16x8 (&pb)[FA_NT]) {
        // V fragments are read three tiles ahead of the MFMAs that use them
        bf16x8 vf[4];
#pragma unroll
        for (int mt = 0; mt < 3; ++mt) vf[mt] = *reinterpret_cast<const bf16x8*>(sp + K_BYTES + (mt * 64 + lane) * 16);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            if (mt + 3 < MT) vf[(mt + 3) & 3] = *reinterpret_cast<const bf16x8*>(sp + K_BYTES + ((mt + 3) * 64 + lane) * 16);
#pragma unroll
            for (int nt = 0; nt < FA_NT; ++nt)
                oacc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[mt & 3], pb[nt], oacc[mt][nt], 0, 0, 0);
        }
#pragma unroll
        for (int nt = 0; nt < FA_NT; ++nt) {
            lacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[nt], lacc[nt], 0, 0, 0);
        }
    };
    // softmax update and O^T += V^T P^T for the block whose scores are in `sacc`
    auto finish = [&](const f32x4 (&sacc)[2][FA_NT], const unsigned char* sp, int t0, auto tail_tag) {
        reference(sacc, t0, tail_tag);
        bf16x8 pb[FA_NT];
#pragma unroll
        for (int nt = 0; nt < FA_NT; ++nt)
#pragma unroll
            for (int e = 0; e < 8; ++e) pb[nt][e] = prob(sacc, nt, e, t0, tail_tag);
        pv(sp, pb);
    };
    const std::integral_constant<bool, false> main_tag;
    const std::integral_constant<bool, true> tail_tag;
    // The hot path (this block and the next lie inside the old cache): the score MFMAs of block
    // i+1 and the exponentials of block i do not depend on each other, so they are issued
    // interleaved, two MFMAs per pair of probabilities, and the matrix cores work through the
    // vector part of the softmax.  The scheduling fences keep the compiler from regrouping each
    // kind into a run of its own.
    auto fused = [&](const f32x4 (&cur)[2][FA_NT], f32x4 (&nxt)[2][FA_NT], const unsigned char* sp_cur,
                     const unsigned char* sp_nxt) {
        auto k_frag = [&](int a, int s) {
            return *reinterpret_cast<const bf16x8*>(sp_nxt + ((a * KS + s) * 64 + lane) * 16);
        };
        bf16x8 k0 = k_frag(0, 0), k1 = k_frag(1, 0);           // in flight during the reference check
        reference(cur, 0, main_tag);
        bf16x8 pb[FA_NT];
        constexpr int PER = 8 / KS;                            // probabilities per (s, nt) step
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            bf16x8 n0 = k0, n1 = k1;
            if (s + 1 < KS) {
                n0 = k_frag(0, s + 1);
                n1 = k_frag(1, s + 1);
            }
#pragma unroll
            for (int nt = 0; nt < FA_NT; ++nt) {
                const bf16x8 qf = s < QS_REG ? qreg[nt][s] : q_lds(nt, s);
                const f32x4 zero4 = (f32x4){0.f, 0.f, 0.f, 0.f};
                nxt[0][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, qf, s == 0 ? zero4 : nxt[0][nt], 0, 0, 0);
                nxt[1][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, qf, s == 0 ? zero4 : nxt[1][nt], 0, 0, 0);
                const int e0 = (s * FA_NT + nt) * PER;
#pragma unroll
                for (int u = 0; u < PER; ++u)
                    pb[(e0 + u) / 8][(e0 + u) % 8] = prob(cur, (e0 + u) / 8, (e0 + u) % 8, 0, main_tag);
                __builtin_amdgcn_sched_barrier(0);
            }
            k0 = n0;
            k1 = n1;
        }
        pv(sp_cur, pb);
    };

    __syncthreads();                                       // matches the producer's first barrier
    static_assert(8 % KS == 0, "whole probabilities per interleaving step");
    f32x4 sa[2][FA_NT], sb[2][FA_NT];
    load_q();
    if (live && nblocks > 0) scores(stage[0], sa);
    // one block: softmax + PV of block i (scores in `cur`) and the scores of block i+1 (into
    // `nxt`).  Off the hot path the two teams do the pieces in opposite order, so that the two
    // waves sharing a SIMD want different units after every barrier.
    auto block = [&](f32x4 (&cur)[2][FA_NT], f32x4 (&nxt)[2][FA_NT], int i) {
        if (!(live && i < nblocks)) return;
        const int t0 = t_begin + i * TSTEP;
        const bool has_next = i + 1 < nblocks;
        if (has_next && t0 + TSTEP + 32 <= L) {
            fused(cur, nxt, stage[i % FA_STAGES], stage[(i + 1) % FA_STAGES]);
            return;
        }
        if (team == 0 && has_next) scores(stage[(i + 1) % FA_STAGES], nxt);
        if (t0 + 32 > L) finish(cur, stage[i % FA_STAGES], t0, tail_tag);
        else finish(cur, stage[i % FA_STAGES], t0, main_tag);
        if (team != 0 && has_next) scores(stage[(i + 1) % FA_STAGES], nxt);
    };
    for (int i = 0; i < nblocks_wg; i += 2) {
        block(sa, sb, i);
        __syncthreads();
        if (i + 1 >= nblocks_wg) break;
        block(sb, sa, i + 1);
        __syncthreads();
    }
    if (!live) return;

    const int64_t item = ((int64_t)b * KVH + kvh) * nqg + qg;
    float* __restrict__ o_out = po + (item * nsplit + split) * FA_QROWS * HD;
    float* __restrict__ ml_out = pml + (item * nsplit + split) * FA_QROWS * 2;
#pragma unroll
    for (int nt = 0; nt < FA_NT; ++nt) {
        const int n = nt * 16 + c;
        if (g == 0) { ml_out[n * 2] = m_run[nt]; ml_out[n * 2 + 1] = lacc[nt][0]; }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            *reinterpret_cast<f32x4*>(o_out + (int64_t)n * HD + mt * 16 + 4 * g) = oacc[mt][nt];
    }
}

// -------------------------------------------------------------------------------------
// kernel for prompt blocks (hundreds of rows per stream and more)
//
// There the pass is bound by the matrix cores and the vector unit, not by HBM: a block of 4096
// rows has 16384 query rows per KV head, and every cached token is used by all of them.  So the
// token axis is not split at all: a workgroup of eight waves owns 256 query rows (32 each: with
// 48, the register tile of the kernels above, a 2048-row block gives 176 workgroups for 256
// compute units and is slower), walks the tokens its rows can see once, and writes the
// normalised result itself (no partial results, no merge).  All eight waves multiply; nobody
// is set aside to load: each wave requests its share (1 KB fragment blocks) of every 32-token
// block with direct-to-LDS loads into a ring of six stages, so four blocks are in flight while
// one is multiplied, and the loads cost no registers.  The loads and the waits on them are
// inline assembly with exact counts, as in the many-row GEMM: after the query fragments have
// arrived the kernel issues no other vector memory load until its final stores.  Per block a
// wave runs scores -> softmax -> PV in sequence (the other wave of its SIMD fills the gaps);
// interleaving them inside the wave, or across the two waves of a SIMD, was slower or spilled.
// Workgroups of one KV head get ids 8 apart (one XCD, one L2); the last rows of a block see the
// most tokens and are dispatched first.
// -------------------------------------------------------------------------------------
#define PF_WAVES 8
#define PF_THREADS (64 * PF_WAVES)
#define PF_STAGES 6
#define PF_NT 2             // 16-row query tiles per wave

template <int HD, int NT, typename OT>
__global__ __launch_bounds__(PF_THREADS) void k_attn_prefill(const bf16_t* __restrict__ q,
                                                             const bf16_t* __restrict__ kc,
                                                             const bf16_t* __restrict__ vc,
                                                             const int32_t* __restrict__ kv_len,
                                                             int rows, int H, int KVH, int64_t cap,
                                                             int nqt, int ranges, int g_shift,
                                                             OT* __restrict__ out, int tiled,
                                                             int32_t* __restrict__ flags) {
    constexpr int KS = HD / 32, MT = HD / 16;
    constexpr int WQROWS = 16 * NT;                     // query rows per wave
    constexpr int PF_QROWS = PF_WAVES * WQROWS;         // ... per workgroup
    constexpr int K_BYTES = 2 * KS * 1024, V_BYTES = MT * 1024;
    constexpr int STAGE_BYTES = K_BYTES + V_BYTES;
    constexpr int NLOAD = 2 * KS + MT;                  // 1 KB requests per 32-token block
    constexpr int LD = NLOAD / PF_WAVES;                // ... per wave
    static_assert(NLOAD % PF_WAVES == 0, "every wave issues the same number of requests");
    __shared__ __attribute__((aligned(16))) unsigned char stage[PF_STAGES][STAGE_BYTES];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);   // uniform copy for the request addresses
    const int c = lane & 15, g = lane >> 4;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int range = (slot / nqt) * 8 + xcd;           // (stream, KV head)
    if (range >= ranges) return;                        // whole workgroup, before any barrier
    const int qt = nqt - 1 - slot % nqt;                // heaviest first
    const int kvh = range % KVH, b = range / KVH;
    const int G = H / KVH;
    const int QR = G * rows;
    const int L = kv_len[b];
    const int n_tok = L + rows;
    // causality: nothing beyond the last row of this workgroup is walked
    const int last_row = min(rows - 1, ((qt + 1) * PF_QROWS - 1) / G);
    const int n_lim = L + last_row + 1;
    const int nblocks = (n_lim + 31) / 32;              // >= 1
    const bf16_t* __restrict__ K = kc + ((int64_t)b * KVH + kvh) * cap * HD;
    const bf16_t* __restrict__ V = vc + ((int64_t)b * KVH + kvh) * HD * cap;

    // query fragments: straight from memory into registers, once
    // query row nt*16 + c of this wave is row n0 + nt*16 of the KV head: block row n >> g_shift,
    // head n & (G - 1) of the group (G is a power of two here)
    const int n0 = qt * PF_QROWS + wave * WQROWS + c;
    bf16x8 qreg[NT][KS];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int n = n0 + nt * 16;
        const bf16_t* qp = q + (((int64_t)(b * rows + (n < QR ? n >> g_shift : 0))) * H + kvh * G + (n < QR ? n & (G - 1) : 0)) * HD + g * 8;
#pragma unroll
        for (int s = 0; s < KS; ++s)
            qreg[nt][s] = n < QR ? *reinterpret_cast<const bf16x8*>(qp + s * 32) : (bf16x8){0, 0, 0, 0, 0, 0, 0, 0};
    }
    // they must have arrived before the first counted request below: the compiler waits for a
    // load where its result is first used, which is here
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int s = 0; s < KS; ++s) asm volatile("" : "+v"(qreg[nt][s]));

    // this wave's requests of a block: fragment block id = wave + 8*u; ids below 2*KS are K
    // fragments (a = id / KS, s = id % KS), the others V fragments (mt = id - 2*KS).  Lane
    // (c, g) of a K fragment holds token ktok0 + 4a, elements s*32 + g*8 ..; of a V fragment
    // feature mt*16 + c, tokens 8g ...
    const int ktok0 = 8 * (c >> 2) + (c & 3);
    unsigned voff[LD];
    const bf16_t* sbase[LD];
    int tstep[LD];                                      // elements the uniform base advances per token
#pragma unroll
    for (int u = 0; u < LD; ++u) {
        const int id = wave_s + PF_WAVES * u;
        if (id < 2 * KS) {
            voff[u] = (unsigned)(((ktok0 + 4 * (id / KS)) * HD + g * 8) * 2);
            sbase[u] = K + (id % KS) * 32;
            tstep[u] = HD;
        } else {
            voff[u] = (unsigned)((((id - 2 * KS) * 16 + c) * CS_VBLK + 8 * g) * 2);
            sbase[u] = V;
            tstep[u] = 0;                               // V: the block address is not linear in t0, see issue
        }
    }
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)&stage[0][0];
    // request block blk (clamped: a surplus request re-reads the last block into a stage nobody reads)
    auto issue = [&](int blk, int st) {
        const int t0 = (blk < nblocks ? blk : nblocks - 1) * 32;
#pragma unroll
        for (int u = 0; u < LD; ++u)
            cs_load_to_lds(voff[u],
                           tstep[u] ? sbase[u] + (int64_t)t0 * tstep[u] : sbase[u] + cs_v_index(t0, 0, HD),
                           lds0 + st * STAGE_BYTES + (wave_s + PF_WAVES * u) * 1024);
    };
    // at most `n` of this wave's requests still in flight, then meet the other waves
#define PF_SYNC(n) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(n) : "memory")

    f32x4 oacc[MT][NT], lacc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        lacc[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) oacc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    float m_run[NT], thr[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) m_run[nt] = thr[nt] = -INFINITY;
    const float scale2 = 1.4426950408889634f / sqrtf((float)HD);
    const float inv_scale2 = sqrtf((float)HD) / 1.4426950408889634f;
    const bf16_t one = (bf16_t)1.0f;
    const bf16x8 ones = (bf16x8){one, one, one, one, one, one, one, one};

    // ---- the pieces of one block (the same arithmetic as in k_attn_lds) ----
    auto scores = [&](const unsigned char* sp, f32x4 (&sacc)[2][NT]) {
        auto k_frag = [&](int a, int s) {
            return *reinterpret_cast<const bf16x8*>(sp + ((a * KS + s) * 64 + lane) * 16);
        };
        bf16x8 k0 = k_frag(0, 0), k1 = k_frag(1, 0);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            bf16x8 n0 = k0, n1 = k1;
            if (s + 1 < KS) {
                n0 = k_frag(0, s + 1);
                n1 = k_frag(1, s + 1);
            }
            const f32x4 zero4 = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                sacc[0][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, qreg[nt][s], s == 0 ? zero4 : sacc[0][nt], 0, 0, 0);
                sacc[1][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, qreg[nt][s], s == 0 ? zero4 : sacc[1][nt], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            k0 = n0;
            k1 = n1;
        }
    };
    auto score_of = [&](const f32x4 (&sacc)[2][NT], int nt, int e, int t0, auto tail_tag) {   // e = 4a + j
        constexpr bool TAIL = decltype(tail_tag)::value;
        const float sc = sacc[e >> 2][nt][e & 3];
        return (TAIL && (t0 + 8 * g + e > L + ((n0 + nt * 16) >> g_shift))) ? -INFINITY : sc;
    };
    auto reference = [&](const f32x4 (&sacc)[2][NT], int t0, auto tail_tag) {
        constexpr bool TAIL = decltype(tail_tag)::value;
        bool calm = false;
        if (!TAIL) {
            bool over = false;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const float lm = fmaxf(fmaxf(fmaxf(sacc[0][nt][0], sacc[0][nt][1]), fmaxf(sacc[0][nt][2], sacc[0][nt][3])),
                                       fmaxf(fmaxf(sacc[1][nt][0], sacc[1][nt][1]), fmaxf(sacc[1][nt][2], sacc[1][nt][3])));
                over |= !(lm <= thr[nt]);
            }
            calm = !__any(over);
        }
        if (calm) return;
        bool moved = false;
        float alpha[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            float mx = fmaxf(fmaxf(score_of(sacc, nt, 0, t0, tail_tag), score_of(sacc, nt, 1, t0, tail_tag)),
                             score_of(sacc, nt, 2, t0, tail_tag));
            mx = fmaxf(fmaxf(mx, score_of(sacc, nt, 3, t0, tail_tag)), score_of(sacc, nt, 4, t0, tail_tag));
            mx = fmaxf(fmaxf(mx, score_of(sacc, nt, 5, t0, tail_tag)),
                       fmaxf(score_of(sacc, nt, 6, t0, tail_tag), score_of(sacc, nt, 7, t0, tail_tag)));
            mx = fa_row4_max(mx);
            mx *= scale2;
            const bool up = mx > m_run[nt] + FA_RESCALE_LOG2;
            const float m_new = up ? mx : m_run[nt];
            alpha[nt] = up ? __builtin_amdgcn_exp2f(m_run[nt] - ((m_new == -INFINITY) ? 0.f : m_new)) : 1.0f;
            moved |= up;
            m_run[nt] = m_new;
            thr[nt] = (m_new == -INFINITY) ? -INFINITY : (m_new + FA_RESCALE_LOG2) * inv_scale2;
        }
        if (__any(moved)) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                lacc[nt] *= alpha[nt];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) oacc[mt][nt] *= alpha[nt];
            }
        }
    };
    auto prob = [&](const f32x4 (&sacc)[2][NT], int nt, int e, int t0, auto tail_tag) {
        const float m_safe = (m_run[nt] == -INFINITY) ? 0.f : m_run[nt];
        return (bf16_t)__builtin_amdgcn_exp2f(fmaf(score_of(sacc, nt, e, t0, tail_tag), scale2, -m_safe));
    };
    // dead: the block reaches past the last appended row; cache rows there may hold anything, and
    // 0 * garbage must stay 0
    auto pv = [&](const unsigned char* sp, const bf16x8 (&pb)[NT], int t0, bool dead) {
        bf16x8 vf[4];
        auto v_frag = [&](int mt) {
            bf16x8 v = *reinterpret_cast<const bf16x8*>(sp + K_BYTES + (mt * 64 + lane) * 16);
            if (dead) {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (t0 + 8 * g + j >= n_tok) v[j] = (bf16_t)0.f;
            }
            return v;
        };
#pragma unroll
        for (int mt = 0; mt < 3; ++mt) vf[mt] = v_frag(mt);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            if (mt + 3 < MT) vf[(mt + 3) & 3] = v_frag(mt + 3);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                oacc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[mt & 3], pb[nt], oacc[mt][nt], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            lacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[nt], lacc[nt], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    };
    auto finish = [&](const f32x4 (&sacc)[2][NT], const unsigned char* sp, int t0, auto tail_tag) {
        reference(sacc, t0, tail_tag);
        __builtin_amdgcn_sched_barrier(0);
        bf16x8 pb[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int e = 0; e < 8; ++e) pb[nt][e] = prob(sacc, nt, e, t0, tail_tag);
        __builtin_amdgcn_sched_barrier(0);
        pv(sp, pb, t0, decltype(tail_tag)::value && t0 + 32 > n_tok);
    };
    const std::integral_constant<bool, false> main_tag;
    const std::integral_constant<bool, true> tail_tag;
    // Blocks 0 .. STAGES-2 are requested up front; iteration i requests block i+STAGES-1 into the
    // stage block i-1 has left, works on block i, and ends when block i+1 has landed in every
    // wave's share (its requests are followed by those of the STAGES-2 blocks that may still be
    // in flight then).
    constexpr int INFLIGHT = LD * (PF_STAGES - 2);
#pragma unroll
    for (int j = 0; j < PF_STAGES - 1; ++j) issue(j, j);
    PF_SYNC(INFLIGHT);
    int st_cur = 0, st_req = PF_STAGES - 1;                 // stage of block i; stage of the next request
    // The loop bound and the cache length are taken from a vector register the compiler cannot
    // see through: with provably uniform branches it splits the live ranges of the accumulators
    // at every branch and ends up copying and spilling them (and a spill reload waits on the
    // same counter as the requests); with branches it must treat as divergent, both sides of
    // a branch work in place under the execution mask.
    int vzero;
    asm volatile("v_mov_b32 %0, 0" : "=v"(vzero));
    const int nblocks_v = nblocks + vzero, L_v = L + vzero;
    // this wave's rows see the tokens up to L + row_lo .. L + row_hi: a block entirely below
    // needs no mask (and holds no dead token), a block entirely above is not computed
    const int row_lo = (n0 - c) >> g_shift;
    const int row_hi = min(rows - 1, (n0 - c + WQROWS - 1) >> g_shift);
    f32x4 sa[2][NT];
    for (int i = 0; i < nblocks_v; ++i) {
        issue(i + PF_STAGES - 1, st_req);
        st_req = st_req + 1 == PF_STAGES ? 0 : st_req + 1;
        const int t0 = i * 32;
        if (t0 <= L_v + row_hi) {
            scores(stage[st_cur], sa);
            if (t0 + 31 > L_v + row_lo) finish(sa, stage[st_cur], t0, tail_tag);
            else finish(sa, stage[st_cur], t0, main_tag);
        }
        st_cur = st_cur + 1 == PF_STAGES ? 0 : st_cur + 1;
        PF_SYNC(INFLIGHT);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");        // surplus requests, before the LDS is given up
#undef PF_SYNC

    // out[r][head*HD + d] = O[d] / l: acc[mt][nt][j] holds O of query row nt*16 + c, feature mt*16 + 4g + j
    // (the float16 input of the output projection: saturated at +-65504, reported if it was)
    bool hit = false;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int n = n0 + nt * 16;
        if (n >= QR) continue;
        const int r = b * rows + (n >> g_shift);
        const int col0 = (kvh * G + (n & (G - 1))) * HD + 4 * g;
        const float inv = 1.0f / lacc[nt][0];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int col = col0 + mt * 16;
            const int64_t off = tiled ? cs_xt_index(r, col, H * HD) : (int64_t)r * H * HD + col;
#pragma unroll
            for (int j = 0; j < 4; ++j) fa_store_out(out, off + j, oacc[mt][nt][j] * inv, hit);
        }
    }
    cs_range_report(flags, hit, CS_RANGE_ATTN);
}

// out[r][h*HD + d] = sum_s 2^(m_s - M) O_s[d] / sum_s 2^(m_s - M) l_s  over the splits
#define FA_MAX_SPLIT 64
// Four output columns per lane (16-byte loads of the partials), HD/4 lanes per query row, so a
// 128-thread workgroup merges 512/HD rows.  Every lane derives the split weights of its row
// itself from the (max, sum) pairs (the HD/4 lanes of a row read the same words, which the
// cache broadcasts): no LDS, no barrier, and the same summation order in every lane.
#define FA_MERGE_THREADS 128
template <typename OT>
__global__ __launch_bounds__(FA_MERGE_THREADS) void k_attn_merge(const float* __restrict__ po,
                                                                 const float* __restrict__ pml,
                                                                 int rows, int H, int KVH, int HD,
                                                                 int nqg, int nsplit,
                                                                 OT* __restrict__ out, int tiled,
                                                                 int32_t* __restrict__ flags) {
    const int lpr = HD >> 2;                  // lanes per query row
    const int n = blockIdx.x * (FA_MERGE_THREADS / lpr) + (int)threadIdx.x / lpr;   // row within the KV head: i*G + gq
    const int d = ((int)threadIdx.x % lpr) * 4;
    const int kvh = blockIdx.y, b = blockIdx.z;
    const int G = H / KVH;
    if (n >= G * rows) return;
    const int i = n / G, gq = n % G;
    const int qg = n / FA_QROWS, nl = n % FA_QROWS;
    const int64_t item = ((int64_t)b * KVH + kvh) * nqg + qg;
    const float2* __restrict__ ml = reinterpret_cast<const float2*>(pml) + (item * nsplit * FA_QROWS + nl);
    const float* __restrict__ o = po + (item * nsplit * FA_QROWS + nl) * HD + d;
    // eight splits at a time, all their loads issued before the first is used: with many splits
    // (one stream: 32) and few workgroups this kernel is nothing but load latency
    float M = -INFINITY;
    for (int w0 = 0; w0 < nsplit; w0 += 8) {
        float mx[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) mx[u] = w0 + u < nsplit ? ml[(int64_t)(w0 + u) * FA_QROWS].x : -INFINITY;
#pragma unroll
        for (int u = 0; u < 8; ++u) M = fmaxf(M, mx[u]);
    }
    float den = 0.f;
    f32x4 num = (f32x4){0.f, 0.f, 0.f, 0.f};
    for (int w0 = 0; w0 < nsplit; w0 += 8) {                // same order in every lane
        float2 p[8];
        f32x4 ov[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const bool in = w0 + u < nsplit;
            p[u] = in ? ml[(int64_t)(w0 + u) * FA_QROWS] : make_float2(-INFINITY, 0.f);
            ov[u] = in ? *reinterpret_cast<const f32x4*>(o + (int64_t)(w0 + u) * FA_QROWS * HD)
                       : (f32x4){0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float wgt = (p[u].x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(p[u].x - M);
            den += wgt * p[u].y;
            num += wgt * ov[u];
        }
    }
    const float inv = 1.0f / den;
    const int r = b * rows + i;
    // tiled: the output projection runs the many-row GEMM, which reads fragment order
    const int col = (kvh * G + gq) * HD + d;
    const int64_t off = tiled ? cs_xt_index(r, col, H * HD) : (int64_t)r * H * HD + col;
    bool hit = false;
    if constexpr (std::is_same<OT, f16_t>::value) {       // one 8-byte store
        const f16x4 o = (f16x4){cs_f16_sat(num[0] * inv, hit), cs_f16_sat(num[1] * inv, hit),
                                cs_f16_sat(num[2] * inv, hit), cs_f16_sat(num[3] * inv, hit)};
        *reinterpret_cast<f16x4*>(out + off) = o;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) fa_store_out(out, off + j, num[j] * inv, hit);
    }
    cs_range_report(flags, hit, CS_RANGE_ATTN);
}

bool cs_attention_fuses_rope(const cs_model* m, int rows) {
    return m->fast && (m->cfg.n_heads / m->cfg.n_kv_heads) * rows <= FA_QROWS;
}

int cs_attention_launch(const cs_model* m, cs_kv* kv, int layer, int rows, int64_t len_ub,
                        int for_o_proj, const float* qkv_part, int qkv_nparts, hipStream_t s) {
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
    // layout of the merged output: fragment order if the output projection (d_model outputs)
    // of these B*rows rows runs the many-row GEMM
    const int tiled = for_o_proj && cs_gemm_x_tiled(B * rows, c.d_model) ? 1 : 0;
    const bf16_t* kc = (const bf16_t*)kv->k + layer * per_layer;
    const bf16_t* vc = (const bf16_t*)kv->v + layer * per_layer;
    CS_REQUIRE(!qkv_part || nqg == 1, CS_E_STATE, "fused rotary embedding needs a narrow block");
    int nsplit;
    // prompt blocks: enough query rows per KV head that a workgroup's 256 rows are all used and
    // the token axis need not be split to fill the chip
    const int pf_qrows = PF_WAVES * 16 * PF_NT;
    const int nqt = (int)cs_ceil_div(QR, pf_qrows);
    int g_shift = 0;
    while ((1 << g_shift) < G) ++g_shift;
    if (QR >= 2 * pf_qrows && (1 << g_shift) == G && (int64_t)B * KVH * nqt >= 40 &&
        (int64_t)hd * kv->cap * 2 < ((int64_t)1 << 32)) {
        const int ranges = B * KVH;
        dim3 grid((unsigned)(cs_round_up(ranges, 8) * nqt));
        const int pa = cs_prof_begin(CS_PROF_ATTN, s);
        if (hd == 128)
            k_attn_prefill<128, PF_NT, f16_t><<<grid, PF_THREADS, 0, s>>>((const bf16_t*)m->q, kc, vc, kv->d_len, rows, H, KVH,
                                                                  kv->cap, nqt, ranges, g_shift, (f16_t*)m->xn, tiled, m->range_flags);
        else
            k_attn_prefill<64, PF_NT, f16_t><<<grid, PF_THREADS, 0, s>>>((const bf16_t*)m->q, kc, vc, kv->d_len, rows, H, KVH,
                                                                 kv->cap, nqt, ranges, g_shift, (f16_t*)m->xn, tiled, m->range_flags);
        cs_prof_end(pa, s);
        return cs_launch_ok("k_attn_prefill");
    }
    if (nqg > 1) {
        // wide block: consumers share the K/V stream of one producer wave through LDS
        const int nqgw = (int)cs_ceil_div(nqg, FA_QG);
        nsplit = FA_TEAMS * (int)cs_ceil_div(256, (int64_t)B * KVH * nqgw);
        const int max_split = (int)cs_ceil_div(n_tok_ub, 256);
        if (nsplit > max_split) nsplit = max_split;
        if (nsplit > FA_MAX_SPLIT) nsplit = FA_MAX_SPLIT;
        if (nsplit < 1) nsplit = 1;
        const int Tw = (int)cs_round_up(cs_ceil_div(n_tok_ub, nsplit), 32);
        nsplit = (int)cs_round_up(cs_ceil_div(n_tok_ub, Tw), FA_TEAMS);
        const size_t items = (size_t)B * KVH * nqg * nsplit;
        CS_REQUIRE(items * FA_QROWS * (hd + 2) <= m->attn_part_floats, CS_E_CAPACITY,
                   "attention workspace too small");
        float* po = m->attn_part;
        float* pml = m->attn_part + items * FA_QROWS * hd;
        // one-dimensional grid, decoded in the kernel (XCD-aware order)
        const int ranges = B * KVH * (nsplit / FA_TEAMS);
        dim3 grid((unsigned)(cs_round_up(ranges, 8) * nqgw));
        const int pa = cs_prof_begin(CS_PROF_ATTN, s);
        if (hd == 128)
            k_attn_lds<128><<<grid, FA_LDS_THREADS, 0, s>>>((const bf16_t*)m->q, kc, vc, kv->d_len, rows,
                                                             H, KVH, kv->cap, Tw, nqg, nqgw, nsplit, ranges, po, pml);
        else
            k_attn_lds<64><<<grid, FA_LDS_THREADS, 0, s>>>((const bf16_t*)m->q, kc, vc, kv->d_len, rows,
                                                            H, KVH, kv->cap, Tw, nqg, nqgw, nsplit, ranges, po, pml);
        cs_prof_end(pa, s);
        CS_TRY(cs_launch_ok("k_attn_lds"));
        dim3 mgrid((unsigned)cs_ceil_div(QR, FA_MERGE_THREADS / (hd / 4)), KVH, B);
        const int pm = cs_prof_begin(CS_PROF_ATTN_MERGE, s);
        k_attn_merge<f16_t><<<mgrid, FA_MERGE_THREADS, 0, s>>>(po, pml, rows, H, KVH, hd, nqg, nsplit,
                                                              (f16_t*)m->xn, tiled, m->range_flags);
        cs_prof_end(pm, s);
        return cs_launch_ok("k_attn_merge");
    }
    // The kernel keeps one wave per SIMD (register budget), so one workgroup fills a compute
    // unit: aim at one workgroup per compute unit, at least 128 tokens per wave.
    nsplit = (int)cs_ceil_div(256, (int64_t)B * KVH * nqg);
    const int max_split = (int)cs_ceil_div(n_tok_ub, 4 * 128);
    if (nsplit > max_split) nsplit = max_split;
    if (nsplit > FA_MAX_SPLIT) nsplit = FA_MAX_SPLIT;
    if (nsplit < 1) nsplit = 1;
    const int Tw = (int)cs_round_up(cs_ceil_div(n_tok_ub, (int64_t)nsplit * 4), 32);
    nsplit = (int)cs_ceil_div(n_tok_ub, (int64_t)Tw * 4);
    const size_t items = (size_t)B * KVH * nqg * nsplit;
    const size_t need = items * FA_QROWS * (hd + 2);
    CS_REQUIRE(need <= m->attn_part_floats, CS_E_CAPACITY,
               "attention workspace too small (%zu > %zu floats)", need, m->attn_part_floats);
    float* po = m->attn_part;
    float* pml = m->attn_part + items * FA_QROWS * hd;
    dim3 grid(nsplit * nqg, KVH, B);
    const int pa = cs_prof_begin(CS_PROF_ATTN, s);
    fa_fused_rope fr = {nullptr, 0, 0, nullptr, nullptr, nullptr, nullptr};
    if (qkv_part) {
        fr.qkv = qkv_part;
        fr.nparts = qkv_nparts;
        fr.part_stride = (int64_t)B * rows * (H + 2 * KVH) * hd;
        fr.rope = m->rope;
        fr.kc_w = (bf16_t*)kv->k + layer * per_layer;
        fr.vc_w = (bf16_t*)kv->v + layer * per_layer;
        fr.bias = m->layers[layer].bqkv;
    }
    if (hd == 128)
        k_attn_mfma<128><<<grid, 256, 0, s>>>((const bf16_t*)m->q, kc, vc, kv->d_len, rows, H, KVH,
                                              kv->cap, Tw, nqg, nsplit, po, pml, fr);
    else
        k_attn_mfma<64><<<grid, 256, 0, s>>>((const bf16_t*)m->q, kc, vc, kv->d_len, rows, H, KVH,
                                             kv->cap, Tw, nqg, nsplit, po, pml, fr);
    cs_prof_end(pa, s);
    CS_TRY(cs_launch_ok("k_attn_mfma"));
    dim3 mgrid((unsigned)cs_ceil_div(QR, FA_MERGE_THREADS / (hd / 4)), KVH, B);
    const int pm = cs_prof_begin(CS_PROF_ATTN_MERGE, s);
    k_attn_merge<f16_t><<<mgrid, FA_MERGE_THREADS, 0, s>>>(po, pml, rows, H, KVH, hd, nqg, nsplit,
                                                          (f16_t*)m->xn, tiled, m->range_flags);
    cs_prof_end(pm, s);
    return cs_launch_ok("k_attn_merge");
}
