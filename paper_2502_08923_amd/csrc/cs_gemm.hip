// Projections of the verify pass: Y[R][N] = X[R][K] * W[N][K]^T.
//
// With R = B*(k+1) block rows (88 at batch 8, k = 10) every weight is used R times, far
// below the ~312 flop/byte ridge of MI355X, so these GEMMs are bound by streaming W from
// HBM once.  The tuned kernel therefore treats W as the operand that must never be
// re-read: each wave loads its W rows straight from global memory into MFMA A-operand
// registers (16 B per lane, 64 contiguous bytes per lane per 128-wide K chunk), while the
// small X block is staged through LDS and shared by the four waves of a workgroup.
// v_mfma_f32_16x16x32_bf16 accumulates in float32.  Small-N projections are split along K
// across workgroups; the float32 partial tiles are summed by the consumer kernel in a
// fixed order (deterministic, no atomics).
#include "cs_common.h"

// -------------------------------------------------------------------------------------
// plain reference kernel: one wave per W row, float32 accumulation
// -------------------------------------------------------------------------------------
template <typename XT, typename WT>
__global__ __launch_bounds__(256) void k_gemm_plain(const XT* __restrict__ X,
                                                    const WT* __restrict__ W, float* __restrict__ Y,
                                                    int R, int N, int K) {
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;
    const WT* __restrict__ w = W + (int64_t)n * K;
    for (int r0 = 0; r0 < R; r0 += 8) {
        float acc[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc[u] = 0.f;
        for (int k = lane; k < K; k += 64) {
            const float wv = cs_ld(w, k);
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (r0 + u < R) acc[u] += wv * cs_ld(X, (int64_t)(r0 + u) * K + k);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float t = cs_wave_sum(acc[u]);
            if (lane == 0 && r0 + u < R) Y[(int64_t)(r0 + u) * N + n] = t;
        }
    }
}

// -------------------------------------------------------------------------------------
// tuned bf16 kernel
// -------------------------------------------------------------------------------------
#define GEMM_KC 128                  // K elements per pipeline stage
#define GEMM_LDS_ROW (GEMM_KC * 2 + 16)   // bytes per X row in LDS (padded)

// MT: 16-row W tiles per wave.  NT: 16-row X tiles per workgroup.
// grid.x: W row tiles of 64*MT, grid.y: K splits, grid.z: X row blocks of 16*NT.
template <int MT, int NT, int MODE>
__global__ __launch_bounds__(256) void k_gemm_mfma(const bf16_t* __restrict__ X,
                                                   const bf16_t* __restrict__ W,
                                                   float* __restrict__ Y, bf16_t* __restrict__ act,
                                                   int R, int N, int K, int Ks) {
    __shared__ __attribute__((aligned(16))) unsigned char xs[2][16 * NT * GEMM_LDS_ROW];
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int lrow = lane & 15, g = lane >> 4;
    const int n_wave = (blockIdx.x * 4 + wave) * MT * 16;       // first W row of this wave
    const int k_begin = blockIdx.y * Ks;
    const int k_end = min(K, k_begin + Ks);
    const int nchunks = (k_end - k_begin) / GEMM_KC;
    const int r_base = blockIdx.z * 16 * NT;

    // per-lane W row pointers (rows past N are clamped; their results are never stored)
    const bf16_t* wrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        int n = n_wave + mt * 16 + lrow;
        n = n < N ? n : N - 1;
        wrow[mt] = W + (int64_t)n * K + g * 32;
    }
    // X staging: thread handles NT 16-byte segments per chunk
    int xr_row[NT];
    const bf16_t* xsrc[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        const int idx = i * 256 + tid;
        xr_row[i] = idx >> 4;
        const int r = r_base + xr_row[i];
        xsrc[i] = (r < R) ? X + (int64_t)r * K + (idx & 15) * 8 : nullptr;
    }

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};

    bf16x8 a_next[MT][4];
    bf16x8 xr[NT];
    auto load_w = [&](int kk) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int s = 0; s < 4; ++s)
                a_next[mt][s] = *reinterpret_cast<const bf16x8*>(wrow[mt] + kk + s * 8);
    };
    auto load_x = [&](int kk) {
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            if (xsrc[i]) xr[i] = *reinterpret_cast<const bf16x8*>(xsrc[i] + kk);
            else xr[i] = (bf16x8){0, 0, 0, 0, 0, 0, 0, 0};
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NT; ++i)
            *reinterpret_cast<bf16x8*>(&xs[buf][xr_row[i] * GEMM_LDS_ROW + ((i * 256 + tid) & 15) * 16]) = xr[i];
    };

    if (nchunks > 0) {
        load_w(k_begin);
        load_x(k_begin);
        store_x(0);
    }
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        bf16x8 a_cur[MT][4];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int s = 0; s < 4; ++s) a_cur[mt][s] = a_next[mt][s];
        const bool more = c + 1 < nchunks;
        if (more) {
            load_w(k_begin + (c + 1) * GEMM_KC);
            load_x(k_begin + (c + 1) * GEMM_KC);
        }
        const unsigned char* xb = xs[c & 1];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const bf16x8 b = *reinterpret_cast<const bf16x8*>(
                    xb + (nt * 16 + lrow) * GEMM_LDS_ROW + g * 64 + s * 16);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_cur[mt][s], b, acc[mt][nt], 0, 0, 0);
            }
        }
        if (more) store_x((c + 1) & 1);
        __syncthreads();
    }

    // epilogue.  acc[mt][nt][j] = Y[row r_base + nt*16 + lrow][col n_wave + mt*16 + 4g + j]
    if (MODE == CS_GEMM_STORE) {
        float* __restrict__ y = Y + (int64_t)blockIdx.y * R * N;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int r = r_base + nt * 16 + lrow;
            if (r >= R) continue;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int n = n_wave + mt * 16 + 4 * g;
                if (n < N) *reinterpret_cast<f32x4*>(y + (int64_t)r * N + n) = acc[mt][nt];
            }
        }
    } else {
        // W rows alternate 16 gate rows / 16 up rows of the same 16 FFN channels
        const int F = N / 2;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int r = r_base + nt * 16 + lrow;
            if (r >= R) continue;
#pragma unroll
            for (int mp = 0; mp < MT / 2; ++mp) {
                const int n = n_wave + mp * 32;
                if (n >= N) continue;
                const int f = n / 2 + 4 * g;
                bf16x4 o;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float gt = acc[2 * mp][nt][j], up = acc[2 * mp + 1][nt][j];
                    o[j] = (bf16_t)(gt / (1.0f + __expf(-gt)) * up);
                }
                *reinterpret_cast<bf16x4*>(act + (int64_t)r * F + f) = o;
            }
        }
    }
}

template <int MT, int NT>
static int launch_mfma(const bf16_t* X, const bf16_t* W, float* Y, bf16_t* act, int R, int N, int K,
                       int mode, int ksplit, hipStream_t s) {
    const int Ks = (int)cs_round_up(cs_ceil_div(K, ksplit), GEMM_KC);
    dim3 grid((unsigned)cs_ceil_div(N, 64 * MT), (unsigned)cs_ceil_div(K, Ks),
              (unsigned)cs_ceil_div(R, 16 * NT));
    const int pg = cs_prof_begin(CS_PROF_GEMM, s);
    if (mode == CS_GEMM_STORE)
        k_gemm_mfma<MT, NT, CS_GEMM_STORE><<<grid, 256, 0, s>>>(X, W, Y, act, R, N, K, Ks);
    else
        k_gemm_mfma<MT, NT, CS_GEMM_SWIGLU><<<grid, 256, 0, s>>>(X, W, Y, act, R, N, K, Ks);
    cs_prof_end(pg, s);
    return cs_launch_ok("k_gemm_mfma");
}

static bool mfma_shape_ok(int N, int K) { return K % GEMM_KC == 0 && N % 16 == 0; }

int cs_gemm_launch(const cs_model* m, const void* X, const void* W, float* Y, int R, int N, int K,
                   int mode, int allow_split, int* nparts_out, hipStream_t s) {
    if (nparts_out) *nparts_out = 1;
    if (R <= 0) return CS_OK;
    if (!m->fast) {
        if (m->cfg.dtype == CS_BF16)
            k_gemm_plain<float, bf16_t><<<(unsigned)cs_ceil_div(N, 4), 256, 0, s>>>(
                (const float*)X, (const bf16_t*)W, Y, R, N, K);
        else
            k_gemm_plain<float, float><<<(unsigned)cs_ceil_div(N, 4), 256, 0, s>>>(
                (const float*)X, (const float*)W, Y, R, N, K);
        return cs_launch_ok("k_gemm_plain");
    }
    if (!mfma_shape_ok(N, K) || (mode == CS_GEMM_SWIGLU && N % 32 != 0)) {
        CS_REQUIRE(mode == CS_GEMM_STORE, CS_E_UNSUPPORTED, "SwiGLU projection needs d_ff %% 16 == 0");
        k_gemm_plain<bf16_t, bf16_t><<<(unsigned)cs_ceil_div(N, 4), 256, 0, s>>>(
            (const bf16_t*)X, (const bf16_t*)W, Y, R, N, K);
        return cs_launch_ok("k_gemm_plain");
    }
    // Split K until there are about two workgroups per compute unit, keeping at least four
    // K chunks per split so the load pipeline has something to overlap.
    const int MT = 2;
    const int n_tiles = (int)cs_ceil_div(N, 64 * MT);
    const int r_blocks = (int)cs_ceil_div(R, 96);
    int ksplit = 1;
    if (allow_split && mode == CS_GEMM_STORE) {
        const int max_split = K / (4 * GEMM_KC) > 0 ? K / (4 * GEMM_KC) : 1;
        while (n_tiles * r_blocks * ksplit < 512 && ksplit * 2 <= max_split) ksplit *= 2;
        while (ksplit > 1 && (size_t)ksplit * R * N > m->part_floats) ksplit /= 2;
    }
    const int Ks = (int)cs_round_up(cs_ceil_div(K, ksplit), GEMM_KC);
    const int nparts = (int)cs_ceil_div(K, Ks);
    if (nparts_out) *nparts_out = nparts;
    const int rt = (int)cs_ceil_div(R < 96 ? R : 96, 16);
    const bf16_t* x = (const bf16_t*)X;
    const bf16_t* w = (const bf16_t*)W;
    bf16_t* act = (bf16_t*)m->act;
    switch (rt) {
        case 1: return launch_mfma<2, 1>(x, w, Y, act, R, N, K, mode, nparts, s);
        case 2: return launch_mfma<2, 2>(x, w, Y, act, R, N, K, mode, nparts, s);
        case 3: return launch_mfma<2, 3>(x, w, Y, act, R, N, K, mode, nparts, s);
        case 4: return launch_mfma<2, 4>(x, w, Y, act, R, N, K, mode, nparts, s);
        case 5: return launch_mfma<2, 5>(x, w, Y, act, R, N, K, mode, nparts, s);
        default: return launch_mfma<2, 6>(x, w, Y, act, R, N, K, mode, nparts, s);
    }
}

int cs_gemm_plain_launch(int dtype, const float* X, const void* W, float* Y, int R, int N, int K,
                         hipStream_t s) {
    if (R <= 0) return CS_OK;
    if (dtype == CS_BF16)
        k_gemm_plain<float, bf16_t><<<(unsigned)cs_ceil_div(N, 4), 256, 0, s>>>(X, (const bf16_t*)W, Y,
                                                                              R, N, K);
    else
        k_gemm_plain<float, float><<<(unsigned)cs_ceil_div(N, 4), 256, 0, s>>>(X, (const float*)W, Y,
                                                                             R, N, K);
    return cs_launch_ok("k_gemm_plain");
}
