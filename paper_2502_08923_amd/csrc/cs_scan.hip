// gamma-gram match scan and draft gather (Sec. 3.1-3.2, App. B.1, App. B.3 step 1).
//
// The paper keeps a hash map of all gamma-grams; on a GPU a linear scan of the int32
// history returns the same position at 4 bytes per token, streamed once.  The scan is
// HBM-bound: every thread loads 16 bytes (4 tokens) per step, compares them with the first
// token of the query suffix, and only on a hit (rare for real vocabularies) checks the
// other gamma-1 tokens.  Each workgroup reduces its chunk to one key; a second tiny
// kernel reduces the chunks of a stream, applies the policy and copies the draft.
//
// Keys (int64, -1 = no candidate): the position for the rightmost (max) and first (min)
// policies; (context length << 32) | position, reduced by max, for the context policy, which
// ranks candidates by how many tokens before them agree with the tokens before the suffix
// (the match-selection refinement the paper's Limitations section leaves open) and takes the
// rightmost among equals.
#include <map>
#include <mutex>
#include <utility>

#include "cs_common.h"

#define SCAN_THREADS 256
#define SCAN_CHUNK 4096   // candidate positions per workgroup
#define SCAN_CONTEXT_CAP 64

// Tokens before candidate p that equal the tokens before the suffix, counted backwards up to
// SCAN_CONTEXT_CAP = 64: the whole wave compares one position per lane, so the length is the
// number of trailing ones of one ballot.  Must be called by all 64 lanes with the same p.
__device__ __forceinline__ int context_length_wave(const int32_t* __restrict__ h, int p, int n, int gamma,
                                                   int lane) {
    const int i = p - lane - 1;
    const bool same = i >= 0 && h[i] == h[n - gamma - lane - 1];
    const unsigned long long agree = __ballot(same);
    return agree == ~0ull ? SCAN_CONTEXT_CAP : __builtin_ctzll(~agree);
}

template <int POLICY>
__device__ __forceinline__ int64_t key_better(int64_t a, int64_t b) {
    if (POLICY == CS_POLICY_FIRST) return (a < 0) ? b : (b < 0 ? a : (a < b ? a : b));
    return a > b ? a : b;
}

__device__ __forceinline__ bool rest_matches(const int32_t* __restrict__ h, int p, int n, int gamma) {
    for (int j = 1; j < gamma; ++j)
        if (h[p + j] != h[n - gamma + j]) return false;
    return true;
}

// The candidates begin, begin + 1, ... of history h[0..n) in strides of THREADS*16 positions
// (`first` and `step` count such strides): a thread loads 16 bytes (4 tokens) per step, compares
// them with the first token of the suffix and only on a hit checks the other gamma - 1.  Returns
// the thread's best key.  Every lane runs every iteration (positions past the end never hit), so
// the wave stays converged for the cooperative context measurement.
template <int POLICY, int THREADS>
__device__ __forceinline__ int64_t scan_strides(const int32_t* __restrict__ h, int n, int gamma, int vec_ok,
                                                int first, int step) {
    constexpr int STRIDE = THREADS * 16;
    const int cnt = n - 2 * gamma + 1;            // candidate starts are 0 .. cnt-1
    int64_t best = -1;
    const int s0 = cnt > 0 ? h[n - gamma] : 0;
    for (int64_t begin64 = (int64_t)first * STRIDE; begin64 < cnt; begin64 += (int64_t)step * STRIDE) {
        const int begin = (int)begin64;
        const int end = (int)min((int64_t)cnt, begin64 + STRIDE);
        for (int it = 0; it < 4; ++it) {
            const int p = begin + (it * THREADS + (int)threadIdx.x) * 4;
            int t[4];
            if (vec_ok && p + 3 < n) {
                const int4 v = *reinterpret_cast<const int4*>(h + p);
                t[0] = v.x; t[1] = v.y; t[2] = v.z; t[3] = v.w;
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) t[i] = (p + i < n) ? h[p + i] : ~s0;
            }
            int hits = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int pp = p + i;
                if (pp < end && t[i] == s0 && rest_matches(h, pp, n, gamma)) {
                    hits |= 1 << i;
                    if (POLICY != CS_POLICY_CONTEXT) best = key_better<POLICY>(best, (int64_t)pp);
                }
            }
            if (POLICY == CS_POLICY_CONTEXT) {
                const int lane = threadIdx.x & 63;
                unsigned long long pending = __ballot(hits != 0);
                while (pending) {                                   // wave-uniform
                    const int src = __builtin_ctzll(pending);
                    pending &= pending - 1;
                    const int p_src = __shfl(p, src, 64);
                    const int h_src = __shfl(hits, src, 64);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (!((h_src >> i) & 1)) continue;          // wave-uniform
                        const int e = context_length_wave(h, p_src + i, n, gamma, lane);
                        if (lane == src) best = key_better<POLICY>(best, ((int64_t)e << 32) | (p_src + i));
                    }
                }
            }
        }
    }
    return best;
}

// best key of the workgroup (valid in every thread): wave shuffle, then LDS across the waves
template <int POLICY, int THREADS>
__device__ __forceinline__ int64_t scan_block_best(int64_t best) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const int64_t other = __shfl_xor(best, o, 64);
        best = key_better<POLICY>(best, other);
    }
    __shared__ int64_t wave_best[THREADS / CS_WAVE];
    if ((threadIdx.x & 63) == 0) wave_best[threadIdx.x >> 6] = best;
    __syncthreads();
    int64_t r = wave_best[0];
#pragma unroll
    for (int w = 1; w < THREADS / CS_WAVE; ++w) r = key_better<POLICY>(r, wave_best[w]);
    return r;
}

// chunk_best[b][s] = best key among the chunks s, s + gridDim.x, ... of stream b, -1 if none
// (SCAN_CHUNK = SCAN_THREADS * 16 positions per chunk).  A workgroup walks its chunks with a stride
// of the grid width, so every candidate position is visited whatever the number of slots the
// launch was given.
template <int POLICY>
__global__ __launch_bounds__(SCAN_THREADS) void k_scan(const int32_t* __restrict__ hist,
                                                       int64_t stride,
                                                       const int32_t* __restrict__ len, int gamma,
                                                       int vec_ok, int64_t* __restrict__ chunk_best,
                                                       int nslots) {
    static_assert(SCAN_CHUNK == SCAN_THREADS * 16, "chunk size and stride of scan_strides agree");
    const int b = blockIdx.y;
    const int64_t best = scan_strides<POLICY, SCAN_THREADS>(hist + (int64_t)b * stride, len[b], gamma, vec_ok,
                                                            blockIdx.x, nslots);
    const int64_t r = scan_block_best<POLICY, SCAN_THREADS>(best);
    if (threadIdx.x == 0) chunk_best[(int64_t)b * nslots + blockIdx.x] = r;
}

// what follows the search: positions from the key, the draft copied from the history (App. B.1,
// the chunk that follows the match), unused slots -1.  Called by every thread of the workgroup.
__device__ __forceinline__ void gather_draft(const int32_t* __restrict__ h, int n, int gamma, int k, int64_t key,
                                             int b, const int32_t* __restrict__ room,
                                             int32_t* __restrict__ match_pos, int32_t* __restrict__ src_pos,
                                             int32_t* __restrict__ draft, int32_t* __restrict__ draft_len) {
    const int best = key < 0 ? -1 : (int)(key & 0x7fffffff);      // low word: the position
    const int src = best < 0 ? -1 : best + gamma;
    int dl = best < 0 ? 0 : min(k, n - src);
    if (room) dl = min(dl, max(room[b] - 1, 0));   // never draft past the emission budget
    if (threadIdx.x == 0) {
        if (match_pos) match_pos[b] = best;
        if (src_pos) src_pos[b] = src;
        draft_len[b] = dl;
    }
    for (int i = threadIdx.x; i < k; i += blockDim.x) draft[(int64_t)b * k + i] = i < dl ? h[src + i] : -1;
}

// One wave per stream: reduce the chunk results, then copy the draft.
__global__ __launch_bounds__(64) void k_gather(const int32_t* __restrict__ hist, int64_t stride,
                                               const int32_t* __restrict__ len, int gamma, int k,
                                               int policy, const int64_t* __restrict__ chunk_best,
                                               int nchunks, const int32_t* __restrict__ room,
                                               int32_t* __restrict__ match_pos,
                                               int32_t* __restrict__ src_pos,
                                               int32_t* __restrict__ draft,
                                               int32_t* __restrict__ draft_len) {
    const int b = blockIdx.x;
    int64_t key = -1;
    for (int c = threadIdx.x; c < nchunks; c += 64) {
        const int64_t v = chunk_best[(int64_t)b * nchunks + c];
        key = policy == CS_POLICY_FIRST ? key_better<CS_POLICY_FIRST>(key, v) : key_better<CS_POLICY_RIGHTMOST>(key, v);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const int64_t other = __shfl_xor(key, o, 64);
        key = policy == CS_POLICY_FIRST ? key_better<CS_POLICY_FIRST>(key, other) : key_better<CS_POLICY_RIGHTMOST>(key, other);
    }
    gather_draft(hist + (int64_t)b * stride, len[b], gamma, k, key, b, room, match_pos, src_pos, draft, draft_len);
}

// Number of key slots per stream a scan over histories of up to max_len tokens wants (one per
// chunk).  Fewer slots are always correct (the workgroups then walk several chunks each).
int cs_scan_slots(int64_t max_len) { return (int)cs_ceil_div(max_len > 0 ? max_len : 1, SCAN_CHUNK); }

// keys: device scratch of B * nslots int64 (every slot is written by k_scan before k_gather reads
// it, so it needs no clearing).  The caller says where it lives: a cache handle's own buffer, the
// per-stream buffers below, or the static array of the entry point that allocates nothing.
int cs_scan_launch(const int32_t* d_hist, int64_t stride, const int32_t* d_len, int B, int gamma,
                   int k, int policy, int64_t* keys, int nslots, int32_t* d_match_pos, int32_t* d_src_pos,
                   int32_t* d_draft, int32_t* d_draft_len, const int32_t* d_room, hipStream_t s) {
    if (B == 0) return CS_OK;
    CS_REQUIRE(keys && nslots >= 1 && B <= 65535, CS_E_ARG, "scan: no key buffer, or more than 65535 histories");
    const int vec_ok = ((reinterpret_cast<uintptr_t>(d_hist) & 15) == 0) && (stride % 4 == 0);
    dim3 grid(nslots, B);
    const int ps = cs_prof_begin(CS_PROF_SCAN, s);
    if (policy == CS_POLICY_RIGHTMOST)
        k_scan<CS_POLICY_RIGHTMOST><<<grid, SCAN_THREADS, 0, s>>>(d_hist, stride, d_len, gamma, vec_ok, keys, nslots);
    else if (policy == CS_POLICY_FIRST)
        k_scan<CS_POLICY_FIRST><<<grid, SCAN_THREADS, 0, s>>>(d_hist, stride, d_len, gamma, vec_ok, keys, nslots);
    else
        k_scan<CS_POLICY_CONTEXT><<<grid, SCAN_THREADS, 0, s>>>(d_hist, stride, d_len, gamma, vec_ok, keys, nslots);
    cs_prof_end(ps, s);
    CS_TRY(cs_launch_ok("k_scan"));
    k_gather<<<B, 64, 0, s>>>(d_hist, stride, d_len, gamma, k, policy, keys, nslots, d_room,
                              d_match_pos, d_src_pos, d_draft, d_draft_len);
    return cs_launch_ok("k_gather");
}

// Key buffers of the entry point that has no handle to keep one in (cs_find_match_batch_dev): one
// per (device, stream) it was ever called on, so that scans enqueued on different streams never
// share scratch and may overlap; calls on one stream are ordered by the stream.  A buffer is
// allocated on the first call on its stream and replaced (after waiting for that stream only) when
// a later call needs a larger one; buffers live until the process ends.
struct scan_keys { int64_t* p; size_t n; };
static std::mutex g_keys_mu;
static std::map<std::pair<int, hipStream_t>, scan_keys> g_keys;

int cs_scan_stream_keys(size_t need, hipStream_t s, int64_t** out) {
    int dev = 0;
    CS_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(g_keys_mu);
    scan_keys& k = g_keys[std::make_pair(dev, s)];
    if (need > k.n) {
        size_t n = 4096;
        while (n < need) n *= 2;
        if (k.p) {
            CS_HIP(hipStreamSynchronize(s));
            (void)hipFree(k.p);
            k.p = nullptr;
            k.n = 0;
        }
        CS_HIP(hipMalloc(&k.p, n * sizeof(int64_t)));
        k.n = n;
    }
    *out = k.p;
    return CS_OK;
}

// draft gather alone, for callers that bring their own per-chunk keys (the gamma-gram index)
int cs_gather_launch(const int32_t* d_hist, int64_t stride, const int32_t* d_len, int B, int gamma, int k,
                     int policy, const int64_t* d_keys, int nchunks, const int32_t* d_room,
                     int32_t* d_match_pos, int32_t* d_src_pos, int32_t* d_draft, int32_t* d_draft_len,
                     hipStream_t s) {
    if (B == 0) return CS_OK;
    k_gather<<<B, 64, 0, s>>>(d_hist, stride, d_len, gamma, k, policy, d_keys, nchunks, d_room, d_match_pos,
                              d_src_pos, d_draft, d_draft_len);
    return cs_launch_ok("k_gather");
}

// -------------------------------------------------------------------------------------
// cs_find_match_batch_dev for callers that must not allocate: same kernels, the per-chunk keys
// live in a fixed array in the code object's own device memory instead of a hipMalloc'd buffer.
// -------------------------------------------------------------------------------------
#define SCAN_STATIC_KEYS CS_NOALLOC_MAX_CHUNKS
static __device__ __align__(256) int64_t scratch[SCAN_STATIC_KEYS];

// `scratch` above is only a host-side stand-in for the symbol; the array's device address is
// asked for once per device (every device holds its own copy at its own address) and only that
// address is ever handed to a kernel.
#define SCAN_MAX_DEVICES 64
static int64_t* g_scratch_ptr[SCAN_MAX_DEVICES];
static std::mutex g_scratch_mu;

static int scan_static_keys(int64_t** out) {
    int dev = 0;
    CS_HIP(hipGetDevice(&dev));
    CS_REQUIRE(dev >= 0 && dev < SCAN_MAX_DEVICES, CS_E_UNSUPPORTED, "device ordinal %d not supported", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        CS_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        CS_REQUIRE(p, CS_E_DEVICE, "no device address for the static scan scratch");
        g_scratch_ptr[dev] = static_cast<int64_t*>(p);
    }
    *out = g_scratch_ptr[dev];
    return CS_OK;
}

extern "C" int cs_find_match_batch_dev_noalloc(const int32_t* d_hist, int64_t stride, const int32_t* d_len,
                                               int32_t B, int32_t gamma, int32_t k, int32_t policy,
                                               int32_t* d_match_pos, int32_t* d_src_pos, int32_t* d_draft,
                                               int32_t* d_draft_len, void* stream) {
    CS_TRY(cs_check_scan_args(gamma, k, policy));
    CS_REQUIRE(B >= 0, CS_E_ARG, "B must be >= 0");
    if (B == 0) return CS_OK;
    CS_REQUIRE(d_hist && d_len && d_draft_len && (d_draft || k == 0), CS_E_ARG,
               "cs_find_match_batch_dev_noalloc: NULL pointer");
    CS_REQUIRE(stride >= 1 && stride <= CS_MAX_STRIDE, CS_E_ARG, "stride out of range");
    const int nslots = cs_scan_slots(stride);
    CS_REQUIRE(B <= 65535 && (int64_t)B * nslots <= SCAN_STATIC_KEYS, CS_E_CAPACITY,
               "cs_find_match_batch_dev_noalloc: B * ceil(stride / %d) = %lld exceeds the static scratch of %d "
               "chunks (use cs_find_match_batch_dev)", SCAN_CHUNK, (long long)B * nslots, SCAN_STATIC_KEYS);
    int64_t* keys = nullptr;
    CS_TRY(scan_static_keys(&keys));
    return cs_scan_launch(d_hist, stride, d_len, B, gamma, k, policy, keys, nslots, d_match_pos, d_src_pos,
                          d_draft, d_draft_len, nullptr, (hipStream_t)stream);
}
