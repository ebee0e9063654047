// Projections of the verify pass: Y[R][N] = X[R][K] * W[N][K]^T.
//
// With R = B*(k+1) block rows (88 at batch 8, k = 10) every weight is used R times, far
// below the ~312 flop/byte ridge of MI355X, so these GEMMs are bound by streaming W from
// HBM once.  The tuned kernel therefore treats W as the operand that must never be
// re-read: each consumer wave loads its W tiles straight from global memory into MFMA
// A-operand registers (W is pre-tiled so that a wave load is 1 KB contiguous), while the
// small X block is staged through LDS by producer waves and shared by the consumers.
// Operands are float16 (weights converted exactly from bfloat16 when the model is created,
// activations rounded to float16 by their producers); v_mfma_f32_16x16x32_f16 accumulates
// in float32.  Small-N projections are split along K across workgroups; the float32 partial
// tiles are summed by the consumer kernel in a fixed order (deterministic, no atomics).
// With hundreds of block rows (large k, large batches, prompt blocks) the same projections
// become compute-bound and go to a second kernel, k_gemm_dma below, that tiles for operand
// reuse and feeds both operands through LDS with direct-to-LDS loads.
#include "cs_common.h"
#include <type_traits>

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
// tuned kernel (fp16 operands, fp32 accumulation)
// -------------------------------------------------------------------------------------
#define GEMM_KC 128                       // K elements per pipeline stage
#define GEMM_LDS_ROW (GEMM_KC * 2 + 16)   // bytes per X row in LDS (padded)
#define GEMM_RING_TILES 8                 // W tile-chunks (4 KB each) in flight per consumer wave
#define GEMM_THREADS 384                  // 4 consumer waves + 2 producer waves

// The workgroup is specialised by wave.  Waves 0..3 (consumers) stream W: each owns MT
// 16-row tiles, keeps 8/MT K-chunks of them (32 KB) in flight in registers and multiplies.
// Waves 4 and 5 (producers) stage the X block of every chunk (half of its rows each)
// through registers into a double-buffered LDS tile.  The hardware counts outstanding loads per wave and retires
// them in order, so a wave that waits for a near X load would also drain its far W loads;
// giving X its own wave keeps the W stream deep.  One barrier per chunk hands the LDS
// buffers over.
// MT: 16-row W tiles per consumer wave.  NT: 16-row X tiles per workgroup.
// grid.x: (W row tile of 64*MT, X row block of 16*NT) pairs, see the mapping below;
// grid.y: K splits.
// act_tiled by mode: SWIGLU - the output goes out in fragment order; ARGMAX - tiles per row of the
// pair buffer.
#define GEMM_STORE_STREAM 3   // CS_GEMM_STORE whose partial tiles leave through streaming stores
template <int MT, int NT, int MODE>
__global__ __launch_bounds__(GEMM_THREADS) void k_gemm_mfma(const f16_t* __restrict__ X,
                                                            const f16_t* __restrict__ W,
                                                            float* __restrict__ Y,
                                                            f16_t* __restrict__ act, int R, int N,
                                                            int K, int Ks, int RB, int act_tiled) {
    __shared__ __attribute__((aligned(16))) unsigned char xs[2][16 * NT * GEMM_LDS_ROW];
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int k_begin = blockIdx.y * Ks;
    const int k_end = min(K, k_begin + Ks);
    const int nchunks = (k_end - k_begin) / GEMM_KC;
    // Workgroup -> (W tile, X row block).  Consecutive workgroup ids go to different XCDs
    // (8 of them, each with its own L2), so the RB row blocks that share one W tile are given
    // ids 8 apart: they run on the same XCD at about the same time and all but the first read
    // W from that L2 instead of HBM.
    const int grp = blockIdx.x / (8 * RB), rem = blockIdx.x % (8 * RB);
    const int w_tile = grp * 8 + (rem & 7);
    if (w_tile * 64 * MT >= N) return;                    // whole workgroup, before any barrier
    const int r_base = (rem >> 3) * 16 * NT;

    if (wave >= 4) {
        // ---------------- producers: X chunks -> LDS ----------------
        // lane -> 16-byte segment (lane & 15) of rows row0 + 4*i, i < ROWS4; the two producer
        // waves split the 16*NT rows in halves
        constexpr int ROWS4 = 2 * NT;
        const int seg = lane & 15, row0 = (lane >> 4) + (wave - 4) * 8 * NT;
        const f16_t* xbase = X + (int64_t)(r_base + row0) * K + k_begin + seg * 8;
        const int64_t xstep = (int64_t)4 * K;
        const int rows_left = R - r_base - row0;          // row 4*i is valid iff 4*i < rows_left
        const int dst0 = row0 * GEMM_LDS_ROW + seg * 16;
        f16x8 xr[2][ROWS4];
        // chunk indices are clamped instead of guarded: a surplus load re-reads the last chunk
        // and a surplus store lands in the buffer nobody reads any more, so the loop body is
        // branch-free and the compiler's load counters stay exact
        const int last = nchunks - 1;
        auto load_x = [&](f16x8* dst, int c) {
            c = c < last ? c : last;
#pragma unroll
            for (int i = 0; i < ROWS4; ++i)
                dst[i] = (4 * i < rows_left)
                             ? *reinterpret_cast<const f16x8*>(xbase + i * xstep + c * GEMM_KC)
                             : (f16x8){0, 0, 0, 0, 0, 0, 0, 0};
        };
        auto store_x = [&](const f16x8* src, int buf) {
#pragma unroll
            for (int i = 0; i < ROWS4; ++i)
                *reinterpret_cast<f16x8*>(&xs[buf][dst0 + i * 4 * GEMM_LDS_ROW]) = src[i];
        };
        load_x(xr[0], 0);
        load_x(xr[1], 1);
        store_x(xr[0], 0);
        load_x(xr[0], 2);
        __syncthreads();
        int c = 0;
        for (; c + 1 < nchunks; c += 2) {
            // chunk c+1 lives in xr[1], chunk c+2 in xr[0]
            store_x(xr[1], 1);
            load_x(xr[1], c + 3);
            __syncthreads();
            store_x(xr[0], 0);
            load_x(xr[0], c + 4);
            __syncthreads();
        }
        if (c < nchunks) __syncthreads();
        if (MODE == CS_GEMM_ARGMAX) {                      // the two barriers of the consumers' epilogue
            __syncthreads();
            __syncthreads();
        }
        return;
    }

    // ---------------- consumers: W stream + MFMA ----------------
    const int lrow = lane & 15, g = lane >> 4;
    const int n_wave = (w_tile * 4 + wave) * MT * 16;           // first W row of this wave
    // W is stored in MFMA fragment order, K-chunk major: W_t[k/128][n/16][(k%128)/32][lane][8].
    // The 16-byte piece `lane` of a 1 KB block is exactly that lane's A operand, so every wave
    // load reads 8 whole cache lines, and all workgroups working on the same K chunk read one
    // contiguous slab of N*256 bytes, which spreads evenly over the HBM channels (a row-major
    // W with its power-of-two row pitch makes concurrent workgroups hit the same channels).
    // (row tiles past N are clamped; their results are never stored)
    const f16_t* wtile[MT];
    const int n_tiles = N >> 4;
    const int64_t chunk_stride = (int64_t)n_tiles * 4 * 512;     // elements per K chunk slab
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        int t = (n_wave >> 4) + mt;
        t = t < n_tiles ? t : n_tiles - 1;
        wtile[mt] = W + (k_begin / GEMM_KC) * chunk_stride + (int64_t)t * 4 * 512 + lane * 8;
    }
    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};

    constexpr int GEMM_DEPTH = GEMM_RING_TILES / MT;            // K chunks in flight
    f16x8 a[GEMM_DEPTH][MT][4];
    const int last = nchunks - 1;
    auto load_w = [&](f16x8 (*dst)[4], int c) {
        c = c < last ? c : last;               // clamped, see the producer
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int s = 0; s < 4; ++s)
                dst[mt][s] = *reinterpret_cast<const f16x8*>(wtile[mt] + c * chunk_stride + s * 512);
    };
    auto compute = [&](f16x8 (*src)[4], int buf) {
        const unsigned char* xb = xs[buf];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const f16x8 bfrag = *reinterpret_cast<const f16x8*>(
                    xb + (nt * 16 + lrow) * GEMM_LDS_ROW + s * 64 + g * 16);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(src[mt][s], bfrag, acc[mt][nt], 0, 0, 0);
            }
        }
    };
#pragma unroll
    for (int u = 0; u < GEMM_DEPTH; ++u) load_w(a[u], u);
    __syncthreads();
    int c = 0;
    for (; c + GEMM_DEPTH <= nchunks; c += GEMM_DEPTH) {      // branch-free groups of DEPTH chunks
#pragma unroll
        for (int u = 0; u < GEMM_DEPTH; ++u) {
            compute(a[u], u & 1);
            load_w(a[u], c + u + GEMM_DEPTH);
            __syncthreads();
        }
    }
#pragma unroll
    for (int u = 0; u < GEMM_DEPTH - 1; ++u) {                // remainder, data already in a[u]
        if (c + u < nchunks) {
            compute(a[u], u & 1);
            __syncthreads();
        }
    }

    // epilogue.  acc[mt][nt][j] = Y[row r_base + nt*16 + lrow][col n_wave + mt*16 + 4g + j]
    if (MODE == CS_GEMM_STORE || MODE == GEMM_STORE_STREAM) {
        float* __restrict__ y = Y + (int64_t)blockIdx.y * R * N;
        if constexpr (MT == 2) {
            // The wave's two 16-column tiles are neighbours: lanes 8 rows apart swap one tile each, so
            // that a store instruction covers 8 rows x 128 bytes (whole lines) instead of 16 rows x 64.
            const bool low = lrow < 8;
            const int n = n_wave + (low ? 0 : 16) + 4 * g;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                f32x4 t0, t1;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    t0[j] = __shfl_xor(acc[0][nt][j], 8, 64);
                    t1[j] = __shfl_xor(acc[1][nt][j], 8, 64);
                }
                const int ra = r_base + nt * 16 + (lrow & 7), rb = ra + 8;
                f32x4* pa = reinterpret_cast<f32x4*>(y + (int64_t)ra * N + n);
                f32x4* pb = reinterpret_cast<f32x4*>(y + (int64_t)rb * N + n);
                const f32x4 va = low ? acc[0][nt] : t1, vb = low ? t0 : acc[1][nt];
                if constexpr (MODE == GEMM_STORE_STREAM) {  // see the launcher
                    if (ra < R && n < N) cs_store_stream(pa, va);
                    if (rb < R && n < N) cs_store_stream(pb, vb);
                } else {
                    if (ra < R && n < N) *pa = va;
                    if (rb < R && n < N) *pb = vb;
                }
            }
        } else {
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
        }
    } else if (MODE == CS_GEMM_ARGMAX) {
        // Per row, the largest of this workgroup's 64*MT columns and its column (the lowest on
        // ties): over the lane's own columns in increasing order, over the four lanes that share
        // a row, then over the four waves through LDS (the X buffers are free).  Y carries the
        // pair buffer [R][tiles][2], act_tiled the number of tiles per row.
        int32_t* __restrict__ am = reinterpret_cast<int32_t*>(Y);
        const int nch = act_tiled;
        float* rv = reinterpret_cast<float*>(&xs[0][0]);                 // [4 waves][16*NT rows]
        int* ri = reinterpret_cast<int*>(&xs[0][0]) + 4 * 16 * NT;
        __syncthreads();                                    // every wave is past its last X fragment
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            float bv = -INFINITY;
            int bi = 0x7fffffff;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                if (n_wave + mt * 16 >= N) continue;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float v = acc[mt][nt][j];
                    if (v > bv) { bv = v; bi = n_wave + mt * 16 + 4 * g + j; }
                }
            }
#pragma unroll
            for (int o = 16; o <= 32; o <<= 1) {
                const float ov = __shfl_xor(bv, o, 64);
                const int oi = __shfl_xor(bi, o, 64);
                cs_am_take(bv, bi, ov, oi);
            }
            if (g == 0) {
                rv[wave * 16 * NT + nt * 16 + lrow] = bv;
                ri[wave * 16 * NT + nt * 16 + lrow] = bi;
            }
        }
        __syncthreads();
        if (tid < 16 * NT && r_base + tid < R) {
            float bv = rv[tid];
            int bi = ri[tid];
#pragma unroll
            for (int w = 1; w < 4; ++w) cs_am_take(bv, bi, rv[w * 16 * NT + tid], ri[w * 16 * NT + tid]);
            const int64_t o = ((int64_t)(r_base + tid) * nch + w_tile) * 2;
            am[o] = __float_as_int(bv);
            am[o + 1] = bi;
        }
    } else {
        // W rows alternate 16 gate rows / 16 up rows of the same 16 FFN channels.  The result is
        // the float16 input of the down projection: saturated at +-65504, and reported through the
        // range flags (Y carries their address in this mode)
        const int F = N / 2;
        bool hit = false;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int r = r_base + nt * 16 + lrow;
            if (r >= R) continue;
#pragma unroll
            for (int mp = 0; mp < MT / 2; ++mp) {
                const int n = n_wave + mp * 32;
                if (n >= N) continue;
                const int f = n / 2 + 4 * g;
                f16x4 o;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float gt = acc[2 * mp][nt][j], up = acc[2 * mp + 1][nt][j];
                    o[j] = cs_f16_sat(gt / (1.0f + __expf(-gt)) * up, hit);
                }
                // act_tiled: the down projection runs the many-row GEMM (fragment order)
                *reinterpret_cast<f16x4*>(act + (act_tiled ? cs_xt_index(r, f, F) : (int64_t)r * F + f)) = o;
            }
        }
        cs_range_report(reinterpret_cast<int32_t*>(Y), hit, CS_RANGE_FFN);
    }
}

// -------------------------------------------------------------------------------------
// tuned kernel for many rows (e.g. batch 16 x (k = 32) + 1 = 528 rows)
//
// With hundreds of block rows the projections are bound by the matrix cores and by the
// bandwidth between L2 and the compute units, so the tile is chosen for operand reuse: a
// workgroup of eight waves (4 x 2, two per SIMD so one wave's waits hide behind the other's
// MFMAs) owns a 256 (W rows) x 32*NT (X rows) output tile, each wave 64 x 16*NT.  Both
// operands go through LDS, every element fetched from L2 once per workgroup.  LDS holds them
// in MFMA fragment order (1 KB blocks of 16 rows x 32 k, lane l's 16 bytes at offset 16*l), so
// fragment reads are conflict-free without padding; the pre-tiled W is already stored that
// way in memory.  The operands never pass through registers on their way in: every wave
// issues 16-byte direct-to-LDS loads (lane l's 16 bytes land at the wave-uniform LDS address
// in M0 plus 16*l, so one load fills one fragment block; X is stored in the same order by
// whoever produces it, see cs_gemm_x_tiled).  K advances 32 at a time through a ring of four
// LDS stages.  Chunk c+3 is requested
// while chunk c is multiplied; one barrier per chunk publishes chunk c+1 and frees the stage
// of chunk c-1, and the first fragments of chunk c+1 are read before that chunk's barrier so
// the matrix cores do not drain at the hand-over.
//
// The loads and the waits on them are written as inline assembly: the compiler's own
// bookkeeping would make every LDS read wait for all outstanding direct-to-LDS loads.  This
// kernel issues no other vector memory loads, so the load counter counts exactly the
// requests below and the s_waitcnt immediates are exact.
// -------------------------------------------------------------------------------------
#define TD_KC 32
#define TG_THREADS 512
#define TG_WROWS 256


// XT: 16-row X tiles per workgroup (8..18).  The two wave rows split them as evenly as whole tiles
// allow: wave row 0 takes the first NT0 = ceil(XT/2), wave row 1 the other NT1 = floor(XT/2); with
// XT odd (528 rows in two blocks: 17 tiles) the two waves of a SIMD, one of each row, then multiply
// 4*17 tile pairs per chunk where an even split rounded up would make it 4*18.
template <int XT, int MODE>
__global__ __launch_bounds__(TG_THREADS) void k_gemm_dma(const f16_t* __restrict__ X,
                                                         const f16_t* __restrict__ W,
                                                         float* __restrict__ Y,
                                                         f16_t* __restrict__ act, int R, int N, int K,
                                                         int Ks, int RB, int act_tiled) {
    constexpr int NT0 = (XT + 1) / 2, NT1 = XT / 2;   // X tiles of a wave in wave row 0 / 1
    constexpr int NBLK = 16 + XT;                     // 1 KB blocks per stage: 16 W tiles, then X tiles
    constexpr int XLD = (XT + 7) / 8;                 // X loads per wave per stage (the last may be partial)
    constexpr int LDMIN = 2 + XT / 8;                 // loads every wave issues per stage
    constexpr int STAGE = NBLK * 1024;
    __shared__ __attribute__((aligned(16))) unsigned char lds[4 * STAGE];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wn = wave & 3, wm = wave >> 2;
    const int lrow = lane & 15, g = lane >> 4;
    const int k_begin = blockIdx.y * Ks;              // multiple of 128
    const int k_end = min(K, k_begin + Ks);
    const int nchunks = (k_end - k_begin) / TD_KC;    // multiple of 4
    const int grp = blockIdx.x / (8 * RB), rem = blockIdx.x % (8 * RB);
    const int w_tile = grp * 8 + (rem & 7);
    if (w_tile * TG_WROWS >= N) return;
    const int r_base = (rem >> 3) * 16 * XT;
    const int n_tiles = N >> 4;
    const int64_t chunk_stride = (int64_t)n_tiles * 4 * 512;

    // wave w requests W tiles w, w+8 and X tiles w, w+8, ... of every chunk.  Both operands are
    // stored in fragment order (W: see k_tile_w; X: cs_xt_index), so every request is one 1 KB
    // block: the lane offset is 16*lane for all of them and the block moves the uniform base.
    const unsigned lane16 = lane * 16;
    const int rt_tiles = (R + 15) >> 4;
    const int64_t x_pitch = (int64_t)(K >> 5) * 512;                   // elements per X row tile
    int tw[2], tx[XLD];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int t = w_tile * 16 + wave + 8 * i;
        tw[i] = t < n_tiles ? t : n_tiles - 1;
    }
#pragma unroll
    for (int i = 0; i < XLD; ++i) {
        int j = wave + 8 * i;
        j = j < XT ? j : XT - 1;
        const int t = (r_base >> 4) + j;
        tx[i] = t < rt_tiles ? t : rt_tiles - 1;
    }
    const f16_t* wbase = W + (int64_t)(k_begin / GEMM_KC) * chunk_stride;
    const f16_t* xbase = X + (int64_t)(k_begin / TD_KC) * 512;
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;

    // request number `idx` (0, 1: W blocks; 2..: X blocks) of chunk c into stage sb
    constexpr int NL = 2 + XLD;                       // requests per wave and chunk (the last may be void)
    auto issue_one = [&](int sb, int c, int idx) {
        const unsigned dst = lds0 + sb * STAGE + wave * 1024;
        if (idx < 2) {
            const f16_t* wc = wbase + (int64_t)(c >> 2) * chunk_stride + (c & 3) * 512;
            cs_load_to_lds(lane16, wc + (int64_t)tw[idx] * 2048, dst + 8 * idx * 1024);
        } else {
            const int i = idx - 2;
            const f16_t* xc = xbase + (int64_t)c * 512;
            if (8 * i + 7 < XT || wave + 8 * i < XT)
                cs_load_to_lds(lane16, xc + tx[i] * x_pitch, dst + (16 + 8 * i) * 1024);
        }
    };
    auto issue = [&](int sb, int c) {
#pragma unroll
        for (int idx = 0; idx < NL; ++idx) issue_one(sb, c, idx);
    };
    const unsigned char* a_base = lds + wn * 4 * 1024 + lane * 16;
    const unsigned char* b_base = lds + (16 + wm * NT0) * 1024 + lane * 16;
    auto a_frag = [&](int sb, int mt) { return *reinterpret_cast<const f16x8*>(a_base + sb * STAGE + mt * 1024); };
    auto b_frag = [&](int sb, int nt) { return *reinterpret_cast<const f16x8*>(b_base + sb * STAGE + nt * 1024); };
    const int n_wave = w_tile * TG_WROWS + wn * 64;

    // wait until at most `n` of this wave's loads are outstanding, then meet the other waves.
    // (A plain s_barrier: the workgroup fence of __syncthreads would drain every load in flight.)
#define TD_SYNC(n) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(n) : "memory")

    // Everything a wave does with its NT X tiles: the multiply loop and the epilogue.  Both wave rows
    // run it with their own NT; the requests, the waits and the barriers are the same in both, so
    // the two instantiations stay in step.
    auto body = [&](auto nt_tag) {
        constexpr int NT = decltype(nt_tag)::value;
        const int xt0 = wm * NT0;                        // first X tile of this wave within the block
        f32x4 acc[4][NT];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
        f16x8 a[4], bq[4];

        issue(0, 0);
        issue(1, 1);
        issue(2, 2);
        TD_SYNC(2 * LDMIN);                                        // chunk 0 has landed everywhere
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) a[mt] = a_frag(0, mt);
        bq[0] = b_frag(0, 0);
        bq[1] = b_frag(0, 1);
        bq[2] = b_frag(0, 2);

        // four chunks, one per stage.  TAIL marks the last trip, where nothing more is requested.
        auto trip = [&](int c0, auto tailc) {
            constexpr bool TAIL = decltype(tailc)::value;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                // chunk c+1 (requested two iterations ago) must be in LDS before its first fragments
                // are read at the end of this iteration; only chunk c+2 may still be in flight
                if (TAIL && u >= 2) TD_SYNC(0);
                else TD_SYNC(LDMIN);
                // chunk c+3 goes to the stage of chunk c-1, free since the barrier.  Its requests are
                // spread over the iteration, one after every few MFMA groups: a wave issues in order,
                // so a burst of requests that the memory pipeline takes one at a time would hold
                // back the MFMAs behind it, in all eight waves at once right after the barrier.
                const bool req = !TAIL || u == 0;
                const bool more = !TAIL || u < 3;
                int next_req = 0;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    if (req && next_req < NL && nt == (next_req * NT) / NL) {
                        issue_one((u + 3) & 3, c0 + u + 3, next_req);
                        ++next_req;
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    const int q = u * NT + nt;                        // position in the B fragment stream
                    if (nt + 3 < NT) bq[(q + 3) & 3] = b_frag(u, nt + 3);              // three tiles ahead
                    else if (more) bq[(q + 3) & 3] = b_frag((u + 1) & 3, nt + 3 - NT);
#pragma unroll
                    for (int mt = 0; mt < 4; ++mt) {
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt], bq[q & 3], acc[mt][nt], 0, 0, 0);
                        // an A fragment is replaced by the next chunk's right after its last use
                        if (nt == NT - 1 && more) a[mt] = a_frag((u + 1) & 3, mt);
                    }
                }
            }
        };
        int c0 = 0;
        for (; c0 + 4 < nchunks; c0 += 4) trip(c0, std::false_type{});
        trip(c0, std::true_type{});

        // epilogue: acc[mt][nt][j] = Y[r_base + (xt0 + nt)*16 + lrow][n_wave + mt*16 + 4g + j]
        if (MODE == CS_GEMM_STORE) {
            float* __restrict__ y = Y + (int64_t)blockIdx.y * R * N;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int r = r_base + (xt0 + nt) * 16 + lrow;
                if (r >= R) continue;
#pragma unroll
                for (int mt = 0; mt < 4; ++mt) {
                    const int n = n_wave + mt * 16 + 4 * g;
                    if (n < N) *reinterpret_cast<f32x4*>(y + (int64_t)r * N + n) = acc[mt][nt];
                }
            }
        } else if (MODE == CS_GEMM_ARGMAX) {
            // as in k_gemm_mfma: the largest of the workgroup's 256 columns per row, lowest column on ties
            int32_t* __restrict__ am = reinterpret_cast<int32_t*>(Y);
            const int nch = act_tiled;
            float* rv = reinterpret_cast<float*>(lds);                        // [4 column waves][16*XT rows]
            int* ri = reinterpret_cast<int*>(lds) + 4 * 16 * XT;
            __syncthreads();                                    // every wave is past its last fragment
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                float bv = -INFINITY;
                int bi = 0x7fffffff;
#pragma unroll
                for (int mt = 0; mt < 4; ++mt) {
                    if (n_wave + mt * 16 >= N) continue;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float v = acc[mt][nt][j];
                        if (v > bv) { bv = v; bi = n_wave + mt * 16 + 4 * g + j; }
                    }
                }
#pragma unroll
                for (int o = 16; o <= 32; o <<= 1) {
                    const float ov = __shfl_xor(bv, o, 64);
                    const int oi = __shfl_xor(bi, o, 64);
                    cs_am_take(bv, bi, ov, oi);
                }
                if (g == 0) {
                    rv[wn * 16 * XT + (xt0 + nt) * 16 + lrow] = bv;
                    ri[wn * 16 * XT + (xt0 + nt) * 16 + lrow] = bi;
                }
            }
            __syncthreads();
            if (tid < 16 * XT && r_base + tid < R) {
                float bv = rv[tid];
                int bi = ri[tid];
#pragma unroll
                for (int w = 1; w < 4; ++w) cs_am_take(bv, bi, rv[w * 16 * XT + tid], ri[w * 16 * XT + tid]);
                const int64_t o = ((int64_t)(r_base + tid) * nch + w_tile) * 2;
                am[o] = __float_as_int(bv);
                am[o + 1] = bi;
            }
        } else {
            const int F = N / 2;
            bool hit = false;                                   // as in k_gemm_mfma
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int r = r_base + (xt0 + nt) * 16 + lrow;
                if (r >= R) continue;
#pragma unroll
                for (int mp = 0; mp < 2; ++mp) {
                    const int n = n_wave + mp * 32;
                    if (n >= N) continue;
                    const int f = n / 2 + 4 * g;
                    f16x4 o;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float gt = acc[2 * mp][nt][j], up = acc[2 * mp + 1][nt][j];
                        o[j] = cs_f16_sat(gt / (1.0f + __expf(-gt)) * up, hit);
                    }
                    *reinterpret_cast<f16x4*>(act + (act_tiled ? cs_xt_index(r, f, F) : (int64_t)r * F + f)) = o;
                }
            }
            cs_range_report(reinterpret_cast<int32_t*>(Y), hit, CS_RANGE_FFN);
        }
    };
    if constexpr (NT0 == NT1) {
        body(std::integral_constant<int, NT0>{});
    } else {
        if (wm == 0) body(std::integral_constant<int, NT0>{});
        else body(std::integral_constant<int, NT1>{});
    }
#undef TD_SYNC
}

template <int XT>
static int launch_tile(const f16_t* X, const f16_t* W, float* Y, f16_t* act, int R, int N, int K, int mode,
                       int ksplit, int act_tiled, hipStream_t s) {
    CS_REQUIRE(((int64_t)R + 15) * K < ((int64_t)1 << 31), CS_E_UNSUPPORTED, "R*K too large for the many-row GEMM");
    const int Ks = (int)cs_round_up(cs_ceil_div(K, ksplit), GEMM_KC);
    const int RB = (int)cs_ceil_div(R, 16 * XT);
    dim3 grid((unsigned)(cs_round_up(cs_ceil_div(N, TG_WROWS), 8) * RB), (unsigned)cs_ceil_div(K, Ks));
    const int pg = cs_prof_begin(CS_PROF_GEMM, s);
    if (mode == CS_GEMM_STORE) k_gemm_dma<XT, CS_GEMM_STORE><<<grid, TG_THREADS, 0, s>>>(X, W, Y, act, R, N, K, Ks, RB, act_tiled);
    else if (mode == CS_GEMM_ARGMAX) k_gemm_dma<XT, CS_GEMM_ARGMAX><<<grid, TG_THREADS, 0, s>>>(X, W, Y, act, R, N, K, Ks, RB, act_tiled);
    else k_gemm_dma<XT, CS_GEMM_SWIGLU><<<grid, TG_THREADS, 0, s>>>(X, W, Y, act, R, N, K, Ks, RB, act_tiled);
    cs_prof_end(pg, s);
    return cs_launch_ok("k_gemm_dma");
}

template <int MT, int NT>
static int launch_mfma(const f16_t* X, const f16_t* W, float* Y, f16_t* act, int R, int N, int K,
                       int mode, int ksplit, int act_tiled, hipStream_t s) {
    const int Ks = (int)cs_round_up(cs_ceil_div(K, ksplit), GEMM_KC);
    const int RB = (int)cs_ceil_div(R, 16 * NT);
    dim3 grid((unsigned)(cs_round_up(cs_ceil_div(N, 64 * MT), 8) * RB), (unsigned)cs_ceil_div(K, Ks));
    const int pg = cs_prof_begin(CS_PROF_GEMM, s);
    if (mode == CS_GEMM_STORE) {
        // From about 64 rows on the partial tiles are better sent on at once (88 rows: step -1 %,
        // 168: -0.9 %, 264: -0.3 %); with few rows the readers find them in the caches and a plain
        // store wins (48 rows +0.4 %, one stream of 11 rows +2.5 to +3.6 %).
        if (R >= 64)
            k_gemm_mfma<MT, NT, GEMM_STORE_STREAM><<<grid, GEMM_THREADS, 0, s>>>(X, W, Y, act, R, N, K, Ks, RB, act_tiled);
        else
            k_gemm_mfma<MT, NT, CS_GEMM_STORE><<<grid, GEMM_THREADS, 0, s>>>(X, W, Y, act, R, N, K, Ks, RB, act_tiled);
    } else if (mode == CS_GEMM_ARGMAX) {
        k_gemm_mfma<MT, NT, CS_GEMM_ARGMAX><<<grid, GEMM_THREADS, 0, s>>>(X, W, Y, act, R, N, K, Ks, RB, act_tiled);
    } else {
        if constexpr (MT % 2 == 0)
            k_gemm_mfma<MT, NT, CS_GEMM_SWIGLU><<<grid, GEMM_THREADS, 0, s>>>(X, W, Y, act, R, N, K, Ks, RB, act_tiled);
    }
    cs_prof_end(pg, s);
    return cs_launch_ok("k_gemm_mfma");
}

static bool mfma_shape_ok(int N, int K) { return K % GEMM_KC == 0 && N % 16 == 0; }

// dst[k/128][n/16][(k%128)/32][lane l][8]: lane l (row n%16 = l%16, k-group l/16) holds the 8
// elements W[n][(k/32)*32 + (l/16)*8 ..].  N_total/n_off place a block of rows inside a taller
// matrix (the fused q,k,v projection).  rowmap 0: source row = n.  rowmap 1: rows alternate
// 16 gate rows (src) / 16 up rows (src2).
__global__ void k_tile_w(const bf16_t* __restrict__ src, const bf16_t* __restrict__ src2, int N, int K,
                         int rowmap, int N_total, int n_off, f16_t* __restrict__ dst, int32_t* flags) {
    const int64_t nvec = (int64_t)N * K / 8;
    const int n_tiles = N >> 4, nt_total = N_total >> 4;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < nvec;
         v += (int64_t)gridDim.x * blockDim.x) {
        const int lane = (int)(v & 63);
        const int s = (int)((v >> 6) & 3);
        const int64_t tile = v >> 8;
        const int nt = (int)(tile % n_tiles);
        const int kc = (int)(tile / n_tiles);
        const int n = nt * 16 + (lane & 15);
        const int k = kc * 128 + s * 32 + (lane >> 4) * 8;
        const bf16_t* sp = src + (int64_t)n * K;
        if (rowmap == 1) {
            const int f = (n >> 5) * 16 + (n & 15);
            sp = (((n >> 4) & 1) ? src2 : src) + (int64_t)f * K;
        }
        const int64_t o = ((((int64_t)kc * nt_total + (n_off >> 4) + nt) * 4 + s) * 64 + lane) * 8;
        // bfloat16 -> float16: exact for 2^-17 <= |w| < 65504 (8 significant bits fit the
        // 11-bit significand, subnormals included); smaller magnitudes round to 2^-24 steps
        const bf16x8 wv = *reinterpret_cast<const bf16x8*>(sp + k);
        f16x8 hv;
        bool bad = false;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            hv[j] = (f16_t)(float)wv[j];
            bad |= !(fabsf((float)wv[j]) <= CS_F16_MAX);      // would become inf (or is a NaN)
        }
        *reinterpret_cast<f16x8*>(dst + o) = hv;
        if (bad && flags) atomicOr(flags, CS_RANGE_WEIGHT);
    }
}

int cs_tile_weights_launch(const void* src, const void* src2, int N, int K, int rowmap, int N_total,
                           int n_off, void* dst, int32_t* flags, hipStream_t s) {
    CS_REQUIRE(mfma_shape_ok(N, K) && N_total % 16 == 0 && n_off % 16 == 0, CS_E_UNSUPPORTED,
               "cannot tile a %d x %d matrix", N, K);
    const int64_t nvec = (int64_t)N * K / 8;
    const int blocks = (int)(cs_ceil_div(nvec, 256) < 8192 ? cs_ceil_div(nvec, 256) : 8192);
    k_tile_w<<<blocks, 256, 0, s>>>((const bf16_t*)src, (const bf16_t*)src2, N, K, rowmap, N_total, n_off,
                                    (f16_t*)dst, flags);
    return cs_launch_ok("k_tile_w");
}

bool cs_gemm_x_tiled(int R, int N) { return R > 96 && (cs_ceil_div(N, TG_WROWS) >= 192 || R > 288); }

// f16 [R][K] row-major -> fragment order (cs_xt_index); rows of the last tile beyond R are zero
__global__ void k_tile_x(const f16_t* __restrict__ src, f16_t* __restrict__ dst, int R, int K, int rt_tiles) {
    // (one thread per 8 consecutive k of one row)
    const int64_t n = (int64_t)rt_tiles * 16 * (K / 8);
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int r = (int)(i / (K / 8)), k = (int)(i % (K / 8)) * 8;
        f16x8 v = (f16x8){0, 0, 0, 0, 0, 0, 0, 0};
        if (r < R) v = *reinterpret_cast<const f16x8*>(src + (int64_t)r * K + k);
        *reinterpret_cast<f16x8*>(dst + cs_xt_index(r, k, K)) = v;
    }
}

int cs_tile_x_launch(const void* src, void* dst, int R, int K, hipStream_t s) {
    const int rt_tiles = (int)cs_ceil_div(R, 16);
    const int64_t n = (int64_t)rt_tiles * 16 * (K / 8);
    k_tile_x<<<(unsigned)(cs_ceil_div(n, 256) < 4096 ? cs_ceil_div(n, 256) : 4096), 256, 0, s>>>(
        (const f16_t*)src, (f16_t*)dst, R, K, rt_tiles);
    return cs_launch_ok("k_tile_x");
}

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
    CS_REQUIRE(mfma_shape_ok(N, K) && (mode != CS_GEMM_SWIGLU || N % 32 == 0), CS_E_UNSUPPORTED,
               "bf16 GEMM needs N %% 16 == 0 and K %% 128 == 0 (N=%d K=%d)", N, K);
    // Shape of the launch.  One workgroup (6 waves, ~250 registers) fills a compute unit.  Wide
    // projections (gate/up, lm_head) have enough 128-row tiles.  Narrow ones (q/k/v, o, down)
    // are split along K, but only until about 3/4 of the compute units have a workgroup:
    // measured at the 8B shapes, more splits cost more in partial-tile traffic and fixed
    // per-workgroup latency than they gain in parallelism (q/k/v 4, o 8, down 8 splits).
    // Weight-streaming kernel: a workgroup takes up to 96 block rows; more rows are split into
    // equal row blocks whose workgroups share each W tile through one XCD's L2 (see the mapping
    // in the kernel).  Many-row kernel: 256 W rows x up to 288 block rows per workgroup.  It needs
    // enough 256-row W tiles, or two row blocks of them, to fill the chip: measured inside whole
    // steps at the 8B shapes it wins from 97 rows on for the lm_head (501 tiles) and from 289
    // rows on for every projection (at 168 and 264 rows the q/k/v and gate/up projections,
    // 24 and 112 tiles, are still faster through the weight-streaming kernel).
    const bool tile = cs_gemm_x_tiled(R, N);
    // the SwiGLU epilogue writes the input of the down projection (d_model outputs, same rows)
    int act_tiled = mode == CS_GEMM_SWIGLU && cs_gemm_x_tiled(R, m->cfg.d_model) ? 1 : 0;
    if (mode == CS_GEMM_ARGMAX) {
        // one (value, column) pair per row and workgroup column tile, in place of Y
        CS_REQUIRE(!allow_split && nparts_out, CS_E_STATE, "argmax epilogue: no K split, tile count wanted");
        act_tiled = (int)cs_ceil_div(N, tile ? TG_WROWS : 128);
        Y = reinterpret_cast<float*>(m->am_val_idx);
    }
    if (mode == CS_GEMM_SWIGLU) Y = reinterpret_cast<float*>(m->range_flags);   // see the epilogue
    const int rt_total = (int)cs_ceil_div(R, 16);
    const int r_blocks = tile ? (int)cs_ceil_div(rt_total, 18) : (int)cs_ceil_div(rt_total, 6);
    int ksplit = 1;
    if (allow_split && mode == CS_GEMM_STORE) {
        const int n_tiles = (int)cs_ceil_div(N, tile ? TG_WROWS : 128);
        const int max_split = K / (4 * GEMM_KC) > 0 ? K / (4 * GEMM_KC) : 1;
        while (n_tiles * r_blocks * ksplit < 192 && ksplit * 2 <= max_split) ksplit *= 2;
    }
    // the partial tiles must fit the workspace
    while (ksplit > 1 && (size_t)ksplit * R * N > m->part_floats) ksplit /= 2;
    if (ksplit > 1) CS_REQUIRE(allow_split, CS_E_STATE, "K split without a partial-tile buffer");
    const int Ks = (int)cs_round_up(cs_ceil_div(K, ksplit), GEMM_KC);
    const int nparts = (int)cs_ceil_div(K, Ks);
    if (nparts_out) *nparts_out = mode == CS_GEMM_ARGMAX ? act_tiled : nparts;
    const int rt = (int)cs_ceil_div(rt_total, r_blocks);
    const f16_t* x = (const f16_t*)X;
    const f16_t* w = (const f16_t*)W;
    f16_t* act = (f16_t*)m->act;
    if (tile) {
        switch (rt) {                                // 16-row X tiles per workgroup
            case 9: return launch_tile<9>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);
            case 10: return launch_tile<10>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);
            case 11: return launch_tile<11>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);
            case 12: return launch_tile<12>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);
            case 13: return launch_tile<13>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);
            case 14: return launch_tile<14>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);
            case 15: return launch_tile<15>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);
            case 16: return launch_tile<16>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);
            case 17: return launch_tile<17>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);
            case 18: return launch_tile<18>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);
            default: return launch_tile<8>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);   // up to 128 rows
        }
    }
    switch (rt) {
        case 1: return launch_mfma<2, 1>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);
        case 2: return launch_mfma<2, 2>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);
        case 3: return launch_mfma<2, 3>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);
        case 4: return launch_mfma<2, 4>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);
        case 5: return launch_mfma<2, 5>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);
        default: return launch_mfma<2, 6>(x, w, Y, act, R, N, K, mode, nparts, act_tiled, s);
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
