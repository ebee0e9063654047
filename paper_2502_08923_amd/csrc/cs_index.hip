// Device-resident gamma-gram index: the paper's own data structure (Sec. 3.1: a map from
// every gamma-token subsequence to where it occurs, updated as tokens are appended; App. B.1
// dictionary D, App. B.3 steps 1b and 2d) as an alternative to the linear scan.
//
// One open-addressing table per stream.  A slot is claimed by the first position whose gram
// hashes there (`rep`, compare-and-swap); every later position with the same tokens (verified
// against the history itself, so hash collisions never change a result) folds into the slot's
// `latest` (atomic max) and `first` (atomic min), which makes the contents independent of the
// order in which threads insert.  The index deliberately lags the history: at length n it
// holds the grams that start at p <= n - 2*gamma, exactly the candidates the non-overlap rule
// of App. B.3 step 1c admits, so a lookup needs no filtering: `latest` is the rightmost
// admissible match and `first` the earliest.  Growing the history by e tokens inserts e grams.
#include "cs_common.h"

struct cs_index {
    int B;
    int gamma;
    int64_t max_len;
    int64_t slots;            // power of two, >= 2 * max_len
    int32_t* rep;             // [B][slots] position that claimed the slot, -1 = empty
    int32_t* latest;          // [B][slots]
    int32_t* first;           // [B][slots]
    int32_t* upto;            // [B] grams starting at p < upto[b] are inserted
    int64_t* key;             // [B] lookup result in the scan's key format
};

__device__ __forceinline__ uint32_t gram_hash(const int32_t* __restrict__ h, int p, int gamma) {
    uint64_t x = 0x9E3779B97F4A7C15ull;
    for (int j = 0; j < gamma; ++j) {
        x ^= (uint32_t)h[p + j];
        x *= 0xFF51AFD7ED558CCDull;
        x ^= x >> 32;
    }
    return (uint32_t)x;
}

__device__ __forceinline__ bool gram_equal(const int32_t* __restrict__ h, int a, int b, int gamma) {
    for (int j = 0; j < gamma; ++j)
        if (h[a + j] != h[b + j]) return false;
    return true;
}

__global__ void k_index_clear(int32_t* rep, int32_t* latest, int32_t* first, int64_t n, int32_t* upto, int B) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        rep[i] = -1;
        latest[i] = -1;
        first[i] = 0x7fffffff;
    }
    if (blockIdx.x == 0)
        for (int b = threadIdx.x; b < B; b += blockDim.x) upto[b] = 0;
}

// insert the grams starting at upto[b] .. len[b] - 2*gamma (grid.y = stream)
__global__ __launch_bounds__(256) void k_index_insert(const int32_t* __restrict__ hist, int64_t stride,
                                                      const int32_t* __restrict__ len, int gamma,
                                                      int64_t slots, int32_t* __restrict__ rep,
                                                      int32_t* __restrict__ latest,
                                                      int32_t* __restrict__ first,
                                                      const int32_t* __restrict__ upto) {
    const int b = blockIdx.y;
    const int32_t* __restrict__ h = hist + (int64_t)b * stride;
    const int target = len[b] - 2 * gamma + 1;            // grams 0 .. target-1 belong in the index
    int32_t* r_b = rep + (int64_t)b * slots;
    int32_t* l_b = latest + (int64_t)b * slots;
    int32_t* f_b = first + (int64_t)b * slots;
    const uint32_t mask = (uint32_t)(slots - 1);
    for (int64_t p64 = (int64_t)upto[b] + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p64 < target;
         p64 += (int64_t)gridDim.x * blockDim.x) {
        const int p = (int)p64;
        uint32_t s = gram_hash(h, p, gamma) & mask;
        // at most `slots` probes: the table is at most half full, so an empty slot always exists
        for (int64_t probe = 0; probe < slots; ++probe, s = (s + 1) & mask) {
            int r = r_b[s];
            if (r < 0) {
                const int old = atomicCAS(&r_b[s], -1, p);
                r = old < 0 ? p : old;
            }
            if (r == p || gram_equal(h, r, p, gamma)) {
                atomicMax(&l_b[s], p);
                atomicMin(&f_b[s], p);
                break;
            }
        }
    }
}

// one thread per stream: record the new extent, then look the query suffix up
__global__ void k_index_lookup(const int32_t* __restrict__ hist, int64_t stride, const int32_t* __restrict__ len,
                               int B, int gamma, int policy, int64_t slots, const int32_t* __restrict__ rep,
                               const int32_t* __restrict__ latest, const int32_t* __restrict__ first,
                               int32_t* __restrict__ upto, int64_t* __restrict__ key) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int32_t* __restrict__ h = hist + (int64_t)b * stride;
    const int n = len[b];
    const int target = n - 2 * gamma + 1;
    if (target > upto[b]) upto[b] = target;
    int64_t found = -1;
    if (target > 0) {
        const int32_t* r_b = rep + (int64_t)b * slots;
        const uint32_t mask = (uint32_t)(slots - 1);
        uint32_t s = gram_hash(h, n - gamma, gamma) & mask;
        for (int64_t probe = 0; probe < slots; ++probe, s = (s + 1) & mask) {
            const int r = r_b[s];
            if (r < 0) break;
            if (gram_equal(h, r, n - gamma, gamma)) {
                found = policy == CS_POLICY_FIRST ? first[(int64_t)b * slots + s] : latest[(int64_t)b * slots + s];
                break;
            }
        }
    }
    key[b] = found;
}

extern "C" int cs_index_create(int32_t B, int64_t max_len, int32_t gamma, cs_index** out) {
    CS_REQUIRE(out, CS_E_ARG, "cs_index_create: NULL output");
    *out = nullptr;
    CS_REQUIRE(B >= 1 && B <= 4096, CS_E_ARG, "cs_index_create: B=%d outside 1..4096", B);
    CS_REQUIRE(gamma >= 1 && gamma <= 16, CS_E_ARG, "gamma must be in 1..16 (got %d)", gamma);
    CS_REQUIRE(max_len >= 1 && max_len < ((int64_t)1 << 30), CS_E_ARG, "max_len out of range");
    cs_index* ix = new cs_index();
    ix->B = B;
    ix->gamma = gamma;
    ix->max_len = max_len;
    ix->slots = 64;
    while (ix->slots < 2 * max_len) ix->slots *= 2;
    const size_t n = (size_t)B * ix->slots;
    ix->rep = ix->latest = ix->first = ix->upto = nullptr;
    ix->key = nullptr;
    if (hipMalloc(&ix->rep, n * 4) != hipSuccess || hipMalloc(&ix->latest, n * 4) != hipSuccess ||
        hipMalloc(&ix->first, n * 4) != hipSuccess || hipMalloc(&ix->upto, (size_t)B * 4) != hipSuccess ||
        hipMalloc(&ix->key, (size_t)B * 8) != hipSuccess) {
        cs_set_error("cs_index_create: out of device memory (%zu slots)", n);
        cs_index_destroy(ix);
        return CS_E_DEVICE;
    }
    const int rc = cs_index_reset(ix, nullptr);
    if (rc != CS_OK) {
        cs_index_destroy(ix);
        return rc;
    }
    CS_HIP(hipDeviceSynchronize());
    *out = ix;
    return CS_OK;
}

extern "C" void cs_index_destroy(cs_index* ix) {
    if (!ix) return;
    (void)hipFree(ix->rep);
    (void)hipFree(ix->latest);
    (void)hipFree(ix->first);
    (void)hipFree(ix->upto);
    (void)hipFree(ix->key);
    delete ix;
}

extern "C" int cs_index_reset(cs_index* ix, void* stream) {
    CS_REQUIRE(ix, CS_E_ARG, "cs_index_reset: NULL index");
    const int64_t n = (int64_t)ix->B * ix->slots;
    const int blocks = (int)(cs_ceil_div(n, 256) < 4096 ? cs_ceil_div(n, 256) : 4096);
    k_index_clear<<<blocks, 256, 0, (hipStream_t)stream>>>(ix->rep, ix->latest, ix->first, n, ix->upto, ix->B);
    return cs_launch_ok("k_index_clear");
}

extern "C" int cs_index_find_match_batch_dev(cs_index* ix, const int32_t* d_hist, int64_t stride,
                                             const int32_t* d_len, int64_t max_new_positions, int32_t k,
                                             int32_t policy, int32_t* d_match_pos, int32_t* d_src_pos,
                                             int32_t* d_draft, int32_t* d_draft_len, void* stream) {
    CS_REQUIRE(ix && d_hist && d_len && d_draft_len && (d_draft || k == 0), CS_E_ARG,
               "cs_index_find_match_batch_dev: NULL pointer");
    CS_REQUIRE(k >= 0 && k <= 256, CS_E_ARG, "k must be in 0..256 (got %d)", k);
    CS_REQUIRE(policy == CS_POLICY_RIGHTMOST || policy == CS_POLICY_FIRST, CS_E_UNSUPPORTED,
               "the index answers the rightmost and first policies only (got %d)", policy);
    CS_REQUIRE(stride >= 1 && stride <= ix->max_len, CS_E_ARG,
               "stride %lld exceeds the index's max_len %lld", (long long)stride, (long long)ix->max_len);
    CS_REQUIRE(max_new_positions >= 0, CS_E_ARG, "max_new_positions must be >= 0");
    hipStream_t s = (hipStream_t)stream;
    {
        // the hint only sizes the grid: the kernel's loop inserts every missing gram whatever it is
        const int64_t want = cs_ceil_div(max_new_positions > 0 ? max_new_positions : 1, 256);
        dim3 grid((unsigned)(want < 2048 ? want : 2048), (unsigned)ix->B);
        k_index_insert<<<grid, 256, 0, s>>>(d_hist, stride, d_len, ix->gamma, ix->slots, ix->rep, ix->latest,
                                            ix->first, ix->upto);
        CS_TRY(cs_launch_ok("k_index_insert"));
    }
    k_index_lookup<<<(unsigned)cs_ceil_div(ix->B, 64), 64, 0, s>>>(d_hist, stride, d_len, ix->B, ix->gamma, policy,
                                                                   ix->slots, ix->rep, ix->latest, ix->first,
                                                                   ix->upto, ix->key);
    CS_TRY(cs_launch_ok("k_index_lookup"));
    return cs_gather_launch(d_hist, stride, d_len, ix->B, ix->gamma, k, policy, ix->key, 1, nullptr, d_match_pos,
                            d_src_pos, d_draft, d_draft_len, s);
}
