// Internal declarations shared by the translation units of libcopyspec (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "../../include/copyspec.h"

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16_t;
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define CS_WAVE 64
// longest history row (tokens): positions and their chunk-rounded bounds must fit an int32
#define CS_MAX_STRIDE ((int64_t)0x7fffffff - 8192)

// ---- error plumbing -----------------------------------------------------------------
void cs_set_error(const char* fmt, ...);

#define CS_HIP(call)                                                                      \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess) {                                                           \
            cs_set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, \
                         __LINE__);                                                       \
            return CS_E_DEVICE;                                                           \
        }                                                                                 \
    } while (0)

#define CS_REQUIRE(cond, code, ...)      \
    do {                                 \
        if (!(cond)) {                   \
            cs_set_error(__VA_ARGS__);   \
            return (code);               \
        }                                \
    } while (0)

#define CS_TRY(expr)              \
    do {                          \
        int rc_ = (expr);         \
        if (rc_ != CS_OK) return rc_; \
    } while (0)

static inline int cs_launch_ok(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        cs_set_error("launch of %s failed: %s", what, hipGetErrorString(e));
        return CS_E_DEVICE;
    }
    return CS_OK;
}

static inline int64_t cs_ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline int64_t cs_round_up(int64_t a, int64_t b) { return cs_ceil_div(a, b) * b; }

// ---- event timing of kernel classes (no-ops unless enabled) ----------------------------
int cs_prof_begin(int cls, hipStream_t s);          // returns a slot index or -1
void cs_prof_end(int slot, hipStream_t s);

// ---- handles ------------------------------------------------------------------------
struct cs_layer_dev {
    void* wqkv;    // [(H+2KVH)*hd][d]   rows: q heads, k heads, v heads
    void* wo;      // [d][H*hd]
    void* wgu;     // [2F][d]; row (f/16)*32 + 16*u + f%16 holds gate (u=0) or up (u=1) of f
    void* wd;      // [d][F]
    float* norm1;
    float* norm2;
    float* bqkv;   // [(H+2KVH)*hd] biases of the q, k, v rows, or NULL
};

struct cs_model {
    cs_model_cfg cfg;
    int plain;          // 1: plain kernels everywhere
    int fast;           // 1: the MFMA kernels are in use (GEMM inputs are fp16, q is bf16)
    int R_max;          // max_batch * (max_k + 1)
    int rows_max;       // max_k + 1
    int prefill_rows;   // rows of one prompt block (single stream): max(rows_max, cs_set_prompt_block_rows)
    size_t esz;         // bytes per weight / cache element
    size_t asz;         // bytes per activation element handed to a GEMM
    void* embed;
    void* lm_head;
    float* final_norm;
    cs_layer_dev* layers;   // host array
    unsigned char* layer_loaded;   // host array: the layer's weights have been given
    int layers_loaded, head_loaded;
    // workspace (device)
    float* x;           // [R][d] residual stream
    void* xn;           // [R][max(d, H*hd)] GEMM input (normed rows / attention output)
    void* q;            // [R][H][hd] rotated queries
    float* gu;          // [R][2F]  (plain path only)
    void* act;          // [R][F]
    float* logits;      // [R][V]
    float* part;        // split-K partial sums
    size_t part_floats;
    float* attn_part;   // attention split partials
    size_t attn_part_floats;
    float2* rope;       // [R][hd/2] (cos, sin) of every block row's position
    double* rope_inv_freq;   // [hd/2] rotary frequencies of the model's own (device), or NULL
    int32_t* tok;       // [R] token of every block row
    int32_t* am_val_idx;// argmax partials: [R][chunks] (float bits, idx) pairs
    int32_t* row_argmax;// [R]
    int32_t* draft;     // [B][max_k]   (cs_step scratch)
    int32_t* draft_len; // [B]
    int32_t* match_pos; // [B]
    int32_t* pending;   // [B]
    int32_t* range_flags; // device word: CS_RANGE_* bits raised by producers of float16 GEMM inputs
    int am_chunks;
};

struct cs_kv {
    const cs_model* m;
    int B;
    int64_t cap;        // allocated positions per stream (multiple of 128): the pitch of the caches
    int64_t limit;      // positions a stream may use: the requested capacity rounded up to 64
    void* k;            // [layer][B][KVH][cap][hd]
    void* v;            // [layer][B][KVH][cap/128][hd][128]  (cs_v_index: 128-token blocks, token index contiguous)
    int32_t* d_len;     // device [B]
    int64_t* h_len_ub;  // host [B] upper bound of each length
    int64_t* scan_keys; // device [B][scan_slots]: per-chunk results of the match scan of cs_step
    int scan_slots;
};

// ---- kernels' host launchers (defined in the .hip files) ------------------------------
// scan
int cs_gather_launch(const int32_t* d_hist, int64_t stride, const int32_t* d_len, int B, int gamma, int k,
                     int policy, const int64_t* d_keys, int nchunks, const int32_t* d_room,
                     int32_t* d_match_pos, int32_t* d_src_pos, int32_t* d_draft, int32_t* d_draft_len,
                     hipStream_t s);
int cs_check_scan_args(int gamma, int k, int policy);     // CS_E_ARG with a message, or CS_OK
int cs_scan_slots(int64_t max_len);
int cs_scan_launch(const int32_t* d_hist, int64_t stride, const int32_t* d_len, int B,
                   int gamma, int k, int policy, int64_t* keys, int nslots, int32_t* d_match_pos,
                   int32_t* d_src_pos, int32_t* d_draft, int32_t* d_draft_len,
                   const int32_t* d_room, hipStream_t s);
int cs_scan_stream_keys(size_t need, hipStream_t s, int64_t** out);

// elementwise / small
int cs_embed_launch(const cs_model* m, const int32_t* tok, int R, hipStream_t s);
int cs_rope_table_launch(const cs_model* m, const int32_t* kv_len, int B, int rows, hipStream_t s);
// x[r] += sum of nparts partial tiles (part[p][r][:]) and, if xn_out, xn_out[r] = rmsnorm(x[r])*gain
// (next_N: output width of the GEMM that reads xn_out; it decides the layout of xn_out)
int cs_addnorm_launch(const cs_model* m, const float* part, int nparts,
                      const float* gain, void* xn_out, int R, int next_N, hipStream_t s);
int cs_rope_append_launch(const cs_model* m, cs_kv* kv, int layer, const float* qkv, int nparts,
                          int rows, hipStream_t s);
int cs_swiglu_launch(const cs_model* m, int R, hipStream_t s);
int cs_tokens_launch(const cs_model* m, const int32_t* pending, const int32_t* draft,
                     const int32_t* draft_len, int B, int k, hipStream_t s);
// accept rule, state update from the argmax partials m->am_val_idx[row][nch]
int cs_accept_launch(const cs_model* m, int nch, int B, int k, const int32_t* draft,
                     const int32_t* draft_len, int32_t* accepted, int32_t* next_tok,
                     int32_t* row_argmax_out, int32_t* kv_len, int32_t* hist, int64_t hist_stride,
                     int32_t* hist_len, int32_t* room, hipStream_t s);
int cs_argmax_accept_launch(const cs_model* m, const float* logits, int B, int k, int V,
                            const int32_t* draft, const int32_t* draft_len, int32_t* accepted,
                            int32_t* next_tok, int32_t* row_argmax_out, int32_t* kv_len,
                            int32_t* hist, int64_t hist_stride, int32_t* hist_len,
                            int32_t* room, hipStream_t s);

// GEMM: Y = X * W^T.  mode 0: float32 result [R][N] written to Y (nparts_out tells how many
// split-K partial tiles were written, each [R_stride][N]); mode 1: SwiGLU epilogue into
// m->act (W is the interleaved gate/up matrix); mode 2 (tuned kernels only): nothing is stored
// but, per row and column tile of a workgroup, the largest value and its lowest column, as
// (float bits, column) pairs m->am_val_idx[row][tile] (nparts_out tells the number of tiles):
// the greedy argmax of the lm_head without the logits ever reaching memory.
enum { CS_GEMM_STORE = 0, CS_GEMM_SWIGLU = 1, CS_GEMM_ARGMAX = 2 };
int cs_gemm_launch(const cs_model* m, const void* X, const void* W, float* Y, int R, int N, int K,
                   int mode, int allow_split, int* nparts_out, hipStream_t s);
int cs_gemm_plain_launch(int dtype, const float* X, const void* W, float* Y, int R, int N, int K,
                         hipStream_t s);

// The many-row GEMM kernel reads its activations in MFMA fragment order as well:
// X_t[r/16][k/32][lane = r%16 + 16*((k%32)/8)][k%8] (K = row length, row tiles padded to 16
// rows), so that one direct-to-LDS request is 1 KB of contiguous memory, like a request for W.
// cs_gemm_x_tiled says whether the GEMM of R rows by N outputs runs that kernel; the producer
// of its X (norm, attention merge, SwiGLU epilogue) then writes this layout.  Four consecutive
// k (k % 4 == 0) stay contiguous.
bool cs_gemm_x_tiled(int R, int N);
__host__ __device__ __forceinline__ int64_t cs_xt_index(int r, int k, int K) {
    return ((int64_t)(r >> 4) * (K >> 5) + (k >> 5)) * 512 + (((r & 15) + 16 * ((k & 31) >> 3)) << 3) + (k & 7);
}
// bytes of an f16 activation matrix of R rows by K in that layout
static inline size_t cs_xt_bytes(int64_t R, int64_t K) { return (size_t)((R + 15) / 16) * (K >> 5) * 1024; }
// row-major f16 [R][K] -> that layout (single operations and tests)
int cs_tile_x_launch(const void* src, void* dst, int R, int K, hipStream_t s);

// V cache of one (stream, KV head): element (token t, feature d) of [cap/128][hd][128].  Within a
// block of 128 tokens every feature row is contiguous in the token index (what the PV product's
// A operand wants), and the 128 feature rows of a block are one contiguous 128*hd-element region
// (what the memory system wants: a workgroup walking the tokens reads 32 KB regions instead of
// hd runs a whole cache row apart).
#define CS_VBLK 128
__host__ __device__ __forceinline__ int64_t cs_v_index(int64_t t, int d, int hd) {
    return ((t >> 7) * hd + d) * CS_VBLK + (t & (CS_VBLK - 1));
}

// bf16 weights of the tuned GEMM live in MFMA fragment order (see cs_gemm.hip)
// (flags: device word in which CS_RANGE_WEIGHT is raised if a weight does not fit float16; may be NULL)
int cs_tile_weights_launch(const void* src, const void* src2, int N, int K, int rowmap, int N_total,
                           int n_off, void* dst, int32_t* flags, hipStream_t s);

// attention: reads m->q, writes m->xn (GEMM-input type) as [R][H*hd], or, if for_o_proj, in
// the layout the output projection's GEMM reads
// If qkv_part is not NULL (allowed when cs_attention_fuses_rope(m, rows)), the kernel takes the
// q/k/v projection's partial tiles instead of m->q and does the rotary embedding and the cache
// append itself (no cs_rope_append_launch before it).
bool cs_attention_fuses_rope(const cs_model* m, int rows);
int cs_attention_launch(const cs_model* m, cs_kv* kv, int layer, int rows, int64_t len_ub,
                        int for_o_proj, const float* qkv_part, int qkv_nparts, hipStream_t s);

// conversion helpers
// element type codes for cs_convert_launch
enum { CS_T_F32 = 0, CS_T_BF16 = 1, CS_T_F16 = 2 };
int cs_convert_launch(const void* src, int src_type, void* dst, int dst_type, int64_t n,
                      hipStream_t s);
int cs_fill_i32_launch(int32_t* p, int32_t v, int64_t n, hipStream_t s);

// ---- device helpers -----------------------------------------------------------------
// request 16 bytes per lane from (uniform base + per-lane byte offset) into LDS at lds_addr + 16*lane.
// M0 carries the LDS address.  The compiler reserves M0 and only ever sets it immediately before
// an instruction of its own that reads it, so overwriting it here is safe; it still warns about
// any reserved register in a clobber list, which is silenced for this one statement.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void cs_load_to_lds(unsigned voff, const void* sbase, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_addr) : "m0");
}
#pragma clang diagnostic pop

__device__ __forceinline__ float cs_ld(const float* p, int64_t i) { return p[i]; }
__device__ __forceinline__ float cs_ld(const bf16_t* p, int64_t i) { return (float)p[i]; }
// Streaming store for the split-K partial tiles of the weight-streaming GEMM at 64 rows and more.
// Their reader runs on any XCD, so the lines are of no use in the writer's L2; sent on at once
// they leave the end-of-kernel write-back nothing to flush (headline step 7.96 -> 7.87 ms).
// Measured and not adopted elsewhere: with few rows the readers find the tiles in the caches
// (one stream +3 %), the many-row GEMM's larger tiles gain from being combined in L2 (+4 %),
// normed rows, SwiGLU outputs and attention partials do not change.
__device__ __forceinline__ void cs_store_stream(f32x4* p, f32x4 v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ void cs_st(float* p, int64_t i, float v) { p[i] = v; }
__device__ __forceinline__ void cs_st(bf16_t* p, int64_t i, float v) { p[i] = (bf16_t)v; }
__device__ __forceinline__ float cs_ld(const f16_t* p, int64_t i) { return (float)p[i]; }
__device__ __forceinline__ void cs_st(f16_t* p, int64_t i, float v) { p[i] = (f16_t)v; }

// float32 -> float16 for the inputs of the tuned projections, saturating: a magnitude beyond the
// largest finite float16 (65504) is stored as +-65504 instead of +-inf, and `hit` is raised (also
// for a NaN, which is stored as it is).  In-range values convert exactly as a plain cast does.
#define CS_F16_MAX 65504.0f
__device__ __forceinline__ f16_t cs_f16_sat(float v, bool& hit) {
    const float c = fminf(fmaxf(v, -CS_F16_MAX), CS_F16_MAX);
    hit |= !(fabsf(v) <= CS_F16_MAX);
    return (f16_t)(v != v ? v : c);
}
// a producer that saturated something reports it in the model's range flags (one atomic per lane
// that hit: rare by construction)
__device__ __forceinline__ void cs_range_report(int32_t* flags, bool hit, int bit) {
    if (hit && flags) atomicOr(flags, bit);
}

// running (largest value, lowest index) pair of an argmax
__device__ __forceinline__ void cs_am_take(float& bv, int& bi, float v, int i) {
    if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
}

__device__ __forceinline__ float cs_wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float cs_wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
