// Internal declarations shared by the HIP translation units of libcsd (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <vector>

#include "../../include/csd.h"

typedef uint16_t bf16_t;   // raw bfloat16 bits

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define CSD_WAVE 64

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round-to-nearest-even through the hardware conversion (v_cvt_pk_bf16_f32 on gfx950)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
// two values packed into one dword, a in the low half
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{a, b}, bf16x2_t));
}

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }

// GEMM / attention inputs on the MFMA path are kept as two bf16 planes, hi = bf16(v) and
// lo = bf16(v - hi): the pair carries ~16 significant bits, and the matrix cores multiply the
// exact bf16 weights by both planes.  This keeps the forward within the logit tolerance of an
// exact-arithmetic reference at no cost in HBM traffic (the path is bandwidth-bound).
//
// The bf16 planes that feed the GEMMs are kept fragment by fragment, [k-step][row tile][16 rows][32 columns]
// with `mtp` row tiles per k-step (the padded row capacity / 16, the same for every row width): the matrix
// operand of (row tile, k-step) is then 1 KB of consecutive memory, eight full cache lines per load instead
// of sixteen half-used ones 2 * K bytes apart; lane (t, g) of the operand reads the 16 bytes at (4 t + g) * 16
// of it, and a writer of one row still stores 64 consecutive bytes per k-step.  mtp = 0: plain row-major
// [row][ld] (the queries handed to the attention kernels).  fp32 inputs are row-major.
__device__ __forceinline__ size_t act_tiled_idx(int row, int col, int mtp) {
    return (((size_t)(col >> 5) * mtp + (row >> 4)) << 9) + ((row & 15) << 5) + (col & 31);
}
template <typename TA>
__device__ __forceinline__ void store_act(TA *p, size_t plane, int row, int col, int ld, int mtp, float v);
template <>
__device__ __forceinline__ void store_act<float>(float *p, size_t, int row, int col, int ld, int, float v) {
    p[(size_t)row * ld + col] = v;
}
template <>
__device__ __forceinline__ void store_act<bf16_t>(bf16_t *p, size_t plane, int row, int col, int ld, int mtp, float v) {
    const size_t idx = mtp > 0 ? act_tiled_idx(row, col, mtp) : (size_t)row * ld + col;
    const bf16_t hi = f32_to_bf16(v);
    p[idx] = hi;
    p[idx + plane] = f32_to_bf16(v - bf16_to_f32(hi));
}

// Four consecutive columns (col a multiple of 4: they share a 32-column block) in one store per plane.
template <typename TA>
__device__ __forceinline__ void store_act4(TA *p, size_t plane, int row, int col, int ld, int mtp, f32x4 v);
template <>
__device__ __forceinline__ void store_act4<float>(float *p, size_t, int row, int col, int ld, int, f32x4 v) {
    *reinterpret_cast<f32x4 *>(p + (size_t)row * ld + col) = v;
}
template <>
__device__ __forceinline__ void store_act4<bf16_t>(bf16_t *p, size_t plane, int row, int col, int ld, int mtp, f32x4 v) {
    const size_t idx = mtp > 0 ? act_tiled_idx(row, col, mtp) : (size_t)row * ld + col;
    u32x2 hi, lo;
#pragma unroll
    for (int w = 0; w < 2; w++) {
        const bf16_t h0 = f32_to_bf16(v[2 * w]), h1 = f32_to_bf16(v[2 * w + 1]);
        hi[w] = (uint32_t)h0 | ((uint32_t)h1 << 16);
        lo[w] = (uint32_t)f32_to_bf16(v[2 * w] - bf16_to_f32(h0)) | ((uint32_t)f32_to_bf16(v[2 * w + 1] - bf16_to_f32(h1)) << 16);
    }
    *reinterpret_cast<u32x2 *>(p + idx) = hi;
    *reinterpret_cast<u32x2 *>(p + idx + plane) = lo;
}

// KV cache addressing.  K: [L][Bmax][H][seq_pad][dh];  V is stored transposed in blocks of 32 positions,
// [L][Bmax][H][seq_pad/32][dh][32], so that the P*V contraction reads 8 consecutive keys per lane and the
// V fragments a wave needs of a 32-key tile are one contiguous dh * 64 bytes (whole cache lines: with plain
// [dh][seq_pad] rows every tile used half of each line it touched and the attention kernel fetched 1.5x its
// bytes).  kv_v_idx gives the element index inside a (layer, sequence, head) region.  When kperm is set (MFMA models), the dh
// entries of a K row (and of a query row) are stored in "pair order": 16-entry tile ti holds the 8 entries
// 8ti..8ti+7 of the first half followed by their rotary partners 8ti+dh/2.. of the second half, so that a
// 16-feature MFMA output tile contains whole rotary pairs.  q.k is invariant under a common permutation.
struct KvGeom {
    int Bmax, H, dh, seq_pad, L, kperm;
};
__host__ __device__ inline int rope_perm(int x, int dh, int kperm) {
    if (!kperm) return x;
    const int half = dh / 2, xp = x < half ? x : x - half;
    return 16 * (xp / 8) + (xp % 8) + (x < half ? 0 : 8);
}
__host__ __device__ inline size_t kv_v_idx(const KvGeom &g, int feature, int pos) {
    return ((size_t)(pos >> 5) * g.dh + feature) * 32 + (pos & 31);
}
__host__ __device__ inline size_t kv_head_elems(const KvGeom &g) { return (size_t)g.seq_pad * g.dh; }
__host__ __device__ inline size_t kv_k_off(const KvGeom &g, int l, int b, int hh) {
    return (((size_t)l * g.Bmax + b) * g.H + hh) * kv_head_elems(g);
}
__host__ __device__ inline size_t kv_v_off(const KvGeom &g, int l, int b, int hh) {
    return (size_t)g.L * g.Bmax * g.H * kv_head_elems(g) + kv_k_off(g, l, b, hh);
}

// Workgroup barrier that orders LDS traffic only: global loads already issued (the weight stream)
// stay in flight across it, where __syncthreads() would wait for every outstanding memory operation.
__device__ __forceinline__ void lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// sum over a block of up to 1024 threads; every thread gets the result; `red` holds >= 16 floats
__device__ __forceinline__ float block_sum(float v, float *red) {
    v = wave_sum(v);
    const int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = 0.f;
    for (int i = 0; i < nw; i++) t += red[i];
    return t;
}
__device__ __forceinline__ float block_max(float v, float *red) {
    v = wave_max(v);
    const int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = red[0];
    for (int i = 1; i < nw; i++) t = fmaxf(t, red[i]);
    return t;
}

// ---------------------------------------------------------------------------------- host side

extern thread_local int32_t g_csd_last_hip_error;

#define CSD_HIP(expr)                                   \
    do {                                                \
        hipError_t e__ = (expr);                        \
        if (e__ != hipSuccess) {                        \
            g_csd_last_hip_error = (int32_t)e__;        \
            return CSD_EHIP;                            \
        }                                               \
    } while (0)

#define CSD_LAUNCH_CHECK() CSD_HIP(hipGetLastError())

struct GemmW {
    void *data = nullptr;   // MFMA path: bf16 tiles [N/16][K/32][64 lanes][8]; generic path: row-major [K][N]
    int K = 0, N = 0;
    int S = 1;              // most K splits (partial-sum planes) a launch may use
};

struct LayerW {
    float *attn_norm = nullptr, *ffn_norm = nullptr;
    GemmW qkv, o, gu, down;
    // arch 1 (T5-style decoder): cross-attention norm, query and output projections, and the fused
    // key|value projection of the encoder output (used once per prompt)
    float *cross_norm = nullptr;
    GemmW cq, co, ckv;
};

// How an attention launch sees its keys.  Default: causal over the cache (block row i of a sequence
// with t cached rows sees rows 0 .. t+i).  fixed_nk > 0: every row sees rows 0 .. fixed_nk-1 (cross-
// attention).  rel_bias != null: add rel_bias[bucket[min(query pos - key pos, 127)] * H + head] to the
// scaled score (T5-style relative-position bias; bucket is a 128-entry table, farther keys share entry 127).
// bias_hd: the same values per head and distance, bias_hd[head * 128 + distance], for the kernels that
// fetch them ahead of the scores (one load instead of two dependent ones).
struct AttnMode {
    int fixed_nk = 0;
    const float *rel_bias = nullptr;
    const int32_t *bucket = nullptr;
    const float *bias_hd = nullptr;
    // tree block: per block row, bit j set = block row j is that row or above it in the tree (null: a plain block,
    // where a row sees every row before it)
    const unsigned long long *anc = nullptr;
};

// which keys a block row sees: the cached rows [0, t), and of the block (stored from t on) the rows its mask names
__device__ __forceinline__ bool tree_sees(unsigned long long anc_row, int key, int t) {
    return key < t || (key - t < 64 && ((anc_row >> (key - t)) & 1ull));
}

enum { CSD_PROF_GEMM = 0, CSD_PROF_ATTN = 1, CSD_PROF_OTHER = 2, CSD_PROF_CLASSES = 3 };

struct csd_model {
    csd_model_cfg cfg;
    bool mfma = false;        // bf16 tiles + MFMA GEMMs; otherwise generic kernels on row-major weights
    bool mfma_attn = false;
    int gemm_rs_min_rows = 33;   // blocks of this many rows or more take the GEMM that splits the rows over the waves
    bool kperm = false;       // q / K rows kept in rotary pair order (see KvGeom)
    int hd = 0;               // n_heads * head_dim
    int seq_pad = 0;          // cache rows per sequence, padded to 64
    int m_max = 0;            // max_batch * max_block
    int s_max = 1;            // most K splits of any GEMM
    void *embed = nullptr;    // [V][d] in cfg.dtype, row-major
    float *final_norm = nullptr;
    GemmW lm;
    std::vector<LayerW> layers;
    // scratch (device)
    float *h = nullptr;          // residual stream [m_max][d] fp32
    void *act = nullptr;         // GEMM input rows [m_pad][max(d, F, hd)]: fp32 row-major, or two bf16 planes (hi, lo) stored
                                 // fragment by fragment on the MFMA path (act_tiled_idx)
    int act_mtp = 0;             // row tiles per k-step of that order (m_pad / 16); 0 on the fp32 paths
    void *qbuf = nullptr;        // rotated queries [m_pad][hd] row-major: fp32, or two bf16 planes
    size_t act_plane = 0;        // elements between the hi and lo planes of act
    size_t q_plane = 0;          // ... and of qbuf
    float *part = nullptr;       // split-K partial sums [s_max][m_max][n_max]
    size_t part_floats = 0;      // its capacity
    float *attn_part = nullptr;  // attention partials (MFMA attention)
    float *probs = nullptr;      // [m_max][V] when the caller does not want them
    float2 *rope = nullptr;      // (cos, sin) of the rotary angles of the current call [m_max][head_dim / 2]
    int attn_chunks_max = 0;
    // the forward for blocks of up to 32 rows (csd_chain.hip): one input buffer per GEMM of a layer
    // (two bf16 planes each, fragment order: QKV input, O input, gate|up input, down input) and the sums of
    // squares per (16-feature tile, row) behind the two folded norms
    bool chain_on = false;
    void *x[4] = {nullptr, nullptr, nullptr, nullptr};
    size_t x_plane[4] = {0, 0, 0, 0};    // elements between the hi and lo planes
    float *ssq[2] = {nullptr, nullptr};
    unsigned *attn_cnt = nullptr;        // arrival counters [max_batch][H] of the attention kernel: zero between launches
    float *rstd = nullptr;                    // [m_max] scratch: 1 / rms of every row's residual stream (per-operation forward)
    int32_t *tree_depth = nullptr;            // [m_max] scratch: depth of every row of a tree block
    unsigned long long *tree_anc = nullptr;   // [m_max] scratch: ancestor masks of a tree block
    bool tree_call = false;                   // the forward being enqueued is over a tree block (csd_verify_tree)
    unsigned long long *tail_rec = nullptr;   // [m_max] per-row records of the review that takes every row at once
    unsigned *tail_cnt = nullptr;        // [max_batch] arrival counters of that review: zero between launches
    // arch 1
    int enc_pad = 0;                 // encoder rows padded to 64
    float *rel_bias = nullptr;       // [32][H] fp32
    int32_t *rel_bucket = nullptr;   // [128] bucket of distance n (n >= 127 shares the last entry)
    float *rel_bias_hd = nullptr;    // [H][128]: rel_bias[rel_bucket[n]][h]
    float *trace = nullptr;
    int32_t *review_block = nullptr;  // [max_batch][max_block] block tokens gathered by csd_review_ctx
    // profiling
    bool prof = false;
    std::vector<hipEvent_t> ev;
    std::vector<int> ev_class;
    size_t ev_used = 0;
    double prof_ms[CSD_PROF_CLASSES] = {0, 0, 0};
    int64_t prof_n[CSD_PROF_CLASSES] = {0, 0, 0};
    std::vector<void *> allocs;
};

// The pieces of a model's per-call scratch block (csd_api.hip)
struct ScratchPtrs {
    float *h;
    void *act, *qbuf;
    float *part, *probs;
    float2 *rope;
    float *attn_part;
    void *x[4];
    float *ssq[2];
    unsigned *attn_cnt;
    unsigned long long *tail_rec;   // per block row: (passed, token) of the review that takes every row at once
    unsigned *tail_cnt;      // per sequence: arrival counter of that review, zero between launches
    int32_t *tree_depth;
    unsigned long long *tree_anc;
    float *rstd;
};
size_t csd_scratch_carve(const csd_model *mod, char *base, ScratchPtrs *out);
ScratchPtrs csd_scratch_install(csd_model *mod, const ScratchPtrs &sp);   // returns the pieces in use before

// csd_forward.hip
int32_t csd_forward_enqueue(csd_model *mod, void *kv, const int32_t *tokens, const int32_t *cache_len,
                            int32_t B, int32_t m, float *logits, hipStream_t st);
int32_t csd_pack_weights(csd_model *mod, const void *const *w, hipStream_t st);
int32_t csd_gemm_setup();    // MFMA models, at creation: lets the GEMM kernels use their dynamic LDS
// host only: column tiles per workgroup and K splits the row-split GEMM takes for an N x K matrix and a block of `rows` rows
int32_t csd_rs_plan_host(int32_t N, int32_t K, int32_t rows, size_t part_floats, int32_t *ct, int32_t *S);
size_t csd_self_kv_bytes(const csd_model *mod);     // the self-attention part of the cache (arch 1 appends the cross part)
// csd_chain.hip: forward for blocks of up to 32 rows, epilogues inside the GEMM kernels
int32_t csd_chain_setup();

bool csd_chain_eligible(const csd_model *mod, int32_t B, int32_t m);
int32_t csd_chain_enqueue(csd_model *mod, void *kv, const int32_t *tokens, const int32_t *cache_len, int32_t B, int32_t m,
                          float *logits, hipStream_t st);
// csd_accept.hip
int32_t csd_softmax_enqueue(const float *logits, float *probs, int64_t rows, int32_t V, float temperature,
                            hipStream_t st);
bool csd_review_rows_fits(const float *logits, const float *probs, const float *q, int32_t V);
int32_t csd_review_rows_enqueue(const float *logits, float *probs, unsigned long long *recs, unsigned *counters,
                                float temperature, const float *q, const uint8_t *q_onehot, const int32_t *draft,
                                int32_t draft_stride, const float *u_acc, const float *u_samp, int32_t B, int32_t k, int32_t V,
                                float lenience, int32_t mode, int32_t *n_accepted, int32_t *next_token, hipStream_t st);
int32_t csd_accept_enqueue(const float *p, const float *q, const uint8_t *q_onehot, const int32_t *draft,
                           int32_t draft_stride, const float *u_acc, const float *u_samp, int32_t B, int32_t k,
                           int32_t V, float lenience, int32_t mode, int32_t *n_accepted, int32_t *next_token,
                           hipStream_t st);

// profiling bracket used by the forward driver
struct ProfScope {
    csd_model *m;
    hipStream_t st;
    bool on;
    ProfScope(csd_model *mod, hipStream_t s, int cls);
    ~ProfScope();
};
