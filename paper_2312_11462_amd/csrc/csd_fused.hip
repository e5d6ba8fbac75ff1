// Single-launch review forward for small blocks (M = B*m <= 16 rows): one persistent grid, one
// workgroup per compute unit, walks through every phase of every layer with a device-wide barrier
// between phases, so the weights stream from HBM without kernel boundaries in between.
//
// Phases of a layer (five barriers):
//   1. QKV projection.  Prologue: rmsnorm(h) into LDS as two bf16 planes.  Epilogue: rotate q and k
//      (the projection's output features are tiled in rotary pair order, so a 16-feature MFMA tile
//      holds whole pairs), append K and V to the cache, store q.
//   2. Block attention over the cached prefix: a workgroup takes (sequence, head, 256 keys), its 8
//      waves one 32-key tile each; partial softmax states merge in LDS, then across workgroups by
//      the last one to arrive.
//   3. Output projection; epilogue h += .
//   4. Gate/up projection (prologue rmsnorm(h) into LDS); epilogue f = silu(gate) * up.
//   5. Down projection; epilogue h += .
// A GEMM work item is a group of TG adjacent 16-feature tiles over the whole K; the 8 waves of the
// workgroup split K, reduce through LDS in a fixed order (deterministic) and one wave per tile
// applies the epilogue, so no partial sums ever travel through HBM.
//
// The same phase functions are also launchable one kernel per phase (debugging / comparison).
#include "csd_internal.h"

#define FUSED_THREADS 512
#define FUSED_WAVES 8

enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3 };
enum { PH_EMBED = 0, PH_QKV, PH_ATTN, PH_O, PH_GU, PH_DOWN, PH_LM, PH_TRACE };

struct FusedLayer {
    const u32x4 *qkv, *o, *gu, *down;
    const float *attn_norm, *ffn_norm;
};

struct FusedParams {
    int M, m, B, d, hd, H, dh, F, V, L, seq_pad, Bmax, kperm;
    int kg_max;        // key groups (256 keys each) covered by the attention phase's item list
    int tg_qkv, tg_lm;
    int lds_red_off, lds_rstd_off;
    float eps, scale, theta;
    const int32_t *tokens, *cache_len;
    const bf16_t *embed;
    const FusedLayer *layers;
    const float *final_norm;
    const u32x4 *lm;
    float *h;
    bf16_t *q;
    size_t q_plane;
    bf16_t *act;       // attention output (row stride hd) and SwiGLU output (row stride F), two planes
    size_t act_plane;
    float *cs;         // rotary table [M][dh/2][cos, sin]
    bf16_t *kv;
    float *attn_part;
    unsigned *attn_cnt;
    float *logits;
    unsigned long long *bar;
    unsigned long long bar_base;
    unsigned *err;
    float *trace;
    unsigned long long *ts;   // optional timing marks [mark][workgroup] (100 MHz wall clock), see TS_*
    int ts_slot;              // first mark index of the current phase (set by the persistent kernel)
};

enum { TS_START = 0, TS_PROLOGUE = 1, TS_LOOP = 2, TS_EPILOGUE = 3, TS_BARRIER = 4, TS_PER_PHASE = 5 };
__device__ __forceinline__ void ts_mark(const FusedParams &P, int which) {
    if (P.ts && threadIdx.x == 0) P.ts[(size_t)(P.ts_slot + which) * gridDim.x + blockIdx.x] = wall_clock64();
}

// ------------------------------------------------------------------- coherent device memory

// The grid spans all 8 XCDs and each XCD has its own L2.  Data one workgroup writes for another
// (residual stream, q, attention output, SwiGLU output, rotary table, attention partials, the new
// K/V rows) is written with agent-coherent stores: buffer stores carrying the sc1 cache-policy bit,
// which write through to the memory side, so the device-wide barrier needs no L2 write-back.  The
// barrier ends with an L2 invalidate, after which consumers read that data with ordinary cached loads
// (one fetch per XCD serves all its workgroups).  Data exchanged inside a phase (attention partials
// for the last-arriving workgroup) is read with sc1 loads.  Raw buffers are also bounds-checked by the
// hardware: an out-of-range load returns 0 and an out-of-range store is dropped.
#define CSD_SC1 16

__device__ __forceinline__ __amdgpu_buffer_rsrc_t co_rsrc(const void *p, size_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)(bytes > 0x7FFFFFFFull ? 0x7FFFFFFFull : bytes),
                                             0x00020000);
}
__device__ __forceinline__ u32x4 co_ld128(__amdgpu_buffer_rsrc_t r, int off) {
    return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, CSD_SC1));
}
__device__ __forceinline__ f32x4 co_ld128f(__amdgpu_buffer_rsrc_t r, int off) {
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, CSD_SC1));
}
__device__ __forceinline__ float co_ld32f(__amdgpu_buffer_rsrc_t r, int off) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, CSD_SC1));
}
__device__ __forceinline__ void co_st128(__amdgpu_buffer_rsrc_t r, int off, u32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(v, r, off, 0, CSD_SC1);
}
__device__ __forceinline__ void co_st128f(__amdgpu_buffer_rsrc_t r, int off, f32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, off, 0, CSD_SC1);
}
__device__ __forceinline__ void co_st64(__amdgpu_buffer_rsrc_t r, int off, u32x2 v) {
    __builtin_amdgcn_raw_buffer_store_b64(v, r, off, 0, CSD_SC1);
}
__device__ __forceinline__ void co_st32f(__amdgpu_buffer_rsrc_t r, int off, float v) {
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), r, off, 0, CSD_SC1);
}
__device__ __forceinline__ void co_st16(__amdgpu_buffer_rsrc_t r, int off, bf16_t v) {
    __builtin_amdgcn_raw_buffer_store_b16(v, r, off, 0, CSD_SC1);
}

// ------------------------------------------------------------------------------ grid barrier

// Two-level arrival counter (groups of BAR_GROUP workgroups, then one top counter) so that no single
// address takes 256 serialized atomics.  Counters only grow: the host passes the number of barriers
// completed by earlier launches (bar_base), so nothing is ever reset.  The wait is bounded: when it
// gives up it raises the error flag, which also releases every later wait, so each wave still exits.
#define BAR_GROUP 32
#define BAR_STRIDE 32   /* unsigned long longs between counters: 256 bytes */

__device__ __forceinline__ void grid_barrier(const FusedParams &P, unsigned long long epoch) {
    __syncthreads();            // all of this workgroup's coherent stores have been acknowledged
    if (threadIdx.x == 0) {
        const int G = gridDim.x, grp = blockIdx.x / BAR_GROUP, ngrp = (G + BAR_GROUP - 1) / BAR_GROUP;
        const int gsize = min(BAR_GROUP, G - grp * BAR_GROUP);
        const unsigned long long old =
            __hip_atomic_fetch_add(P.bar + BAR_STRIDE * (1 + grp), 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old + 1 == epoch * (unsigned long long)gsize)
            __hip_atomic_fetch_add(P.bar, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned spins = 0;
        bool give_up = __hip_atomic_load(P.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
        while (!give_up && __hip_atomic_load(P.bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < epoch * (unsigned long long)ngrp) {
            ++spins;
            if ((spins & 1023u) == 0u && __hip_atomic_load(P.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)
                give_up = true;
            if (spins > (1u << 20)) {
                __hip_atomic_store(P.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                give_up = true;
            }
        }
        // drop this XCD's possibly stale lines: data other workgroups wrote (write-through) before the
        // barrier is read with ordinary, L2-cached loads afterwards
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    __syncthreads();
}

// ------------------------------------------------------------------------------------ helpers

__device__ __forceinline__ void split8(const float *v, u32x4 &hi, u32x4 &lo) {
#pragma unroll
    for (int w = 0; w < 4; w++) {
        const uint32_t h = pack_bf16x2(v[2 * w], v[2 * w + 1]);
        hi[w] = h;
        lo[w] = pack_bf16x2(v[2 * w] - __uint_as_float(h << 16), v[2 * w + 1] - __uint_as_float(h & 0xFFFF0000u));
    }
}
__device__ __forceinline__ void split4(const float *v, u32x2 &hi, u32x2 &lo) {
#pragma unroll
    for (int w = 0; w < 2; w++) {
        const uint32_t h = pack_bf16x2(v[2 * w], v[2 * w + 1]);
        hi[w] = h;
        lo[w] = pack_bf16x2(v[2 * w] - __uint_as_float(h << 16), v[2 * w + 1] - __uint_as_float(h & 0xFFFF0000u));
    }
}

// ------------------------------------------------------------------------------------- phases

// h[r] = E[token[r]] and the rotary table of this call's positions
__device__ void phase_embed(const FusedParams &P, int wg, int nwg) {
    const size_t gtid = (size_t)wg * FUSED_THREADS + threadIdx.x, gsz = (size_t)nwg * FUSED_THREADS;
    const __amdgpu_buffer_rsrc_t rh = co_rsrc(P.h, sizeof(float) * (size_t)P.M * P.d);
    const __amdgpu_buffer_rsrc_t rc = co_rsrc(P.cs, sizeof(float) * (size_t)P.M * P.dh);
    const int d8 = P.d / 8;
    for (size_t c = gtid; c < (size_t)P.M * d8; c += gsz) {
        const int r = (int)(c / d8), x8 = (int)(c % d8);
        const int tok = P.tokens[r];
        float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (tok >= 0 && tok < P.V) {
            const u32x4 e = *reinterpret_cast<const u32x4 *>(P.embed + (size_t)tok * P.d + x8 * 8);
#pragma unroll
            for (int w = 0; w < 4; w++) {
                v[2 * w] = __uint_as_float(e[w] << 16);
                v[2 * w + 1] = __uint_as_float(e[w] & 0xFFFF0000u);
            }
        }
        const int off = (int)(((size_t)r * P.d + x8 * 8) * 4);
        co_st128f(rh, off, f32x4{v[0], v[1], v[2], v[3]});
        co_st128f(rh, off + 16, f32x4{v[4], v[5], v[6], v[7]});
    }
    const int half = P.dh / 2;
    for (size_t c = gtid; c < (size_t)P.M * half; c += gsz) {
        const int r = (int)(c / half), x = (int)(c % half);
        const int pos = P.cache_len[r / P.m] + r % P.m;
        const double ang = (double)pos * pow((double)P.theta, -2.0 * (double)x / (double)P.dh);
        co_st32f(rc, (int)(c * 8), (float)cos(ang));
        co_st32f(rc, (int)(c * 8 + 4), (float)sin(ang));
    }
}

// rmsnorm(h) * gain for all M rows into LDS as fragment-ordered hi/lo planes:
// 16-byte unit ((ks*2 + plane)*4 + g)*M + row holds k = 32 ks + 8 g .. +7 of that row.
// One round trip to memory: the fp32 chunk of 8 values is parked in the very two units that later
// receive its hi and lo halves, row sums are taken from LDS, then each thread converts its own units.
__device__ void norm_to_lds(const FusedParams &P, const float *__restrict__ gain, char *smem) {
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int M = P.M, d = P.d, d8 = d / 8;
    float *rstd = reinterpret_cast<float *>(smem + P.lds_rstd_off);
    f32x4 *act = reinterpret_cast<f32x4 *>(smem);
    for (int kc = tid; kc < d8; kc += FUSED_THREADS) {
        const int ks = kc >> 2, g = kc & 3;
        for (int r0 = 0; r0 < M; r0 += 4) {
            f32x4 a[4][2];
#pragma unroll
            for (int u = 0; u < 4; u++)
                if (r0 + u < M) {
                    a[u][0] = *reinterpret_cast<const f32x4 *>(P.h + (size_t)(r0 + u) * d + kc * 8);
                    a[u][1] = *reinterpret_cast<const f32x4 *>(P.h + (size_t)(r0 + u) * d + kc * 8 + 4);
                }
#pragma unroll
            for (int u = 0; u < 4; u++)
                if (r0 + u < M) {
                    act[((ks * 2 + 0) * 4 + g) * M + r0 + u] = a[u][0];
                    act[((ks * 2 + 1) * 4 + g) * M + r0 + u] = a[u][1];
                }
        }
    }
    __syncthreads();
    for (int r = w; r < M; r += FUSED_WAVES) {
        float ss = 0.f;
#pragma unroll 4
        for (int u = lane; u < d8 * 2; u += 64) {          // unit (kc, plane) of row r
            const int kc = u >> 1, pl = u & 1, ks = kc >> 2, g = kc & 3;
            const f32x4 v = act[((ks * 2 + pl) * 4 + g) * M + r];
            ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
        }
        ss = wave_sum(ss);
        if (lane == 0) rstd[r] = rsqrtf(ss / (float)d + P.eps);
    }
    __syncthreads();
    for (int kc = tid; kc < d8; kc += FUSED_THREADS) {
        const int ks = kc >> 2, g = kc & 3;
        const f32x4 g0 = *reinterpret_cast<const f32x4 *>(gain + kc * 8);
        const f32x4 g1 = *reinterpret_cast<const f32x4 *>(gain + kc * 8 + 4);
#pragma unroll 2
        for (int r = 0; r < M; r++) {
            const float rs = rstd[r];
            const int u0 = ((ks * 2 + 0) * 4 + g) * M + r, u1 = ((ks * 2 + 1) * 4 + g) * M + r;
            const f32x4 a0 = act[u0], a1 = act[u1];
            float v[8];
#pragma unroll
            for (int j = 0; j < 4; j++) {
                v[j] = a0[j] * rs * g0[j];
                v[4 + j] = a1[j] * rs * g1[j];
            }
            u32x4 hi, lo;
            split8(v, hi, lo);
            act[u0] = __builtin_bit_cast(f32x4, hi);
            act[u1] = __builtin_bit_cast(f32x4, lo);
        }
    }
    __syncthreads();
}

struct GemmArgs {
    const u32x4 *Wp;       // tiles [n_tiles][KS][64]
    int KS, n_items;       // k-steps of 32; work items (groups of TG tiles)
    const bf16_t *bsrc;    // B operand rows in global memory (two planes) when not from LDS
    size_t bplane;
    int ldb;
    const float *gain;     // norm gain for the LDS prologue
    int layer;
};

template <int TG, int EPI>
__device__ __forceinline__ void gemm_epilogue(const FusedParams &P, const GemmArgs &A, int item, int j, f32x4 v, int lane) {
    const int t = lane & 15, g = lane >> 4;
    const int T = item * TG + j;     // global tile index
    if (EPI == EPI_RESID) {
        const __amdgpu_buffer_rsrc_t rh = co_rsrc(P.h, sizeof(float) * (size_t)P.M * P.d);
        if (t < P.M) {
            const int off = (int)(((size_t)t * P.d + T * 16 + 4 * g) * 4);
            f32x4 cur = *reinterpret_cast<const f32x4 *>(P.h + (size_t)t * P.d + T * 16 + 4 * g);
            cur += v;
            co_st128f(rh, off, cur);
        }
    } else if (EPI == EPI_LOGITS) {
        if (t < P.M) *reinterpret_cast<f32x4 *>(P.logits + (size_t)t * P.V + T * 16 + 4 * g) = v;
    } else if (EPI == EPI_QKV) {
        const int tiles_per_region = P.hd / 16, tiles_per_head = P.dh / 16;
        const int region = T / tiles_per_region, tr = T % tiles_per_region;
        const int head = tr / tiles_per_head, ti = tr % tiles_per_head;
        const int b = t / P.m, pos = (t < P.M) ? P.cache_len[b] + t % P.m : 0;
        const KvGeom geo{P.Bmax, P.H, P.dh, P.seq_pad, P.L, P.kperm};
        const size_t head_bytes = kv_head_elems(geo) * 2;
        if (region < 2) {
            // lanes g < 2 hold first-half entries, lanes g >= 2 their rotary partners (same row, same r)
            float out[4];
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const float other = __shfl_xor(v[r], 32, 64);
                const int xp = 8 * ti + 4 * (g & 1) + r;
                float c = 1.f, s = 0.f;
                if (t < P.M) {
                    c = P.cs[((size_t)t * (P.dh / 2) + xp) * 2];
                    s = P.cs[((size_t)t * (P.dh / 2) + xp) * 2 + 1];
                }
                out[r] = g < 2 ? v[r] * c - other * s : other * s + v[r] * c;
            }
            if (t < P.M) {
                const int p0 = 16 * ti + 4 * g;          // position inside the head, pair order
                if (region == 0) {
                    u32x2 hi, lo;
                    split4(out, hi, lo);
                    const __amdgpu_buffer_rsrc_t rq = co_rsrc(P.q, 2 * (P.q_plane * 2));
                    const int off = (int)(((size_t)t * P.hd + head * P.dh + p0) * 2);
                    co_st64(rq, off, hi);
                    co_st64(rq, off + (int)(P.q_plane * 2), lo);
                } else if (pos >= 0 && pos < P.seq_pad) {
                    u32x2 kk;
                    kk[0] = (uint32_t)f32_to_bf16(out[0]) | ((uint32_t)f32_to_bf16(out[1]) << 16);
                    kk[1] = (uint32_t)f32_to_bf16(out[2]) | ((uint32_t)f32_to_bf16(out[3]) << 16);
                    const __amdgpu_buffer_rsrc_t rk = co_rsrc(P.kv + kv_k_off(geo, A.layer, b, head), head_bytes);
                    co_st64(rk, (int)(((size_t)pos * P.dh + p0) * 2), kk);
                }
            }
        } else if (t < P.M && pos >= 0 && pos < P.seq_pad) {
            const __amdgpu_buffer_rsrc_t rv = co_rsrc(P.kv + kv_v_off(geo, A.layer, b, head), head_bytes);
#pragma unroll
            for (int r = 0; r < 4; r++)
                co_st16(rv, (int)(((size_t)(16 * ti + 4 * g + r) * P.seq_pad + pos) * 2), f32_to_bf16(v[r]));
        }
    }
}

// One weight-streaming GEMM phase.  B_LDS: the B operand (activations) sits in LDS (after norm_to_lds),
// otherwise it is read from the two global planes at A.bsrc.
template <int TG, int EPI, bool B_LDS, int U>
__device__ void gemm_phase(const FusedParams &P, const GemmArgs &A, char *smem, int wg, int nwg) {
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int t = lane & 15, g = lane >> 4;
    const int M = P.M, KS = A.KS;
    const u32x4 *lds_act = reinterpret_cast<const u32x4 *>(smem);
    f32x4 *red = reinterpret_cast<f32x4 *>(smem + P.lds_red_off);
    if (wg >= A.n_items) return;      // whole workgroup idle in this phase (uniform)
    if (B_LDS) norm_to_lds(P, A.gain, smem);
    ts_mark(P, TS_PROLOGUE);
    const int ks0 = KS * w / FUSED_WAVES, ks1 = KS * (w + 1) / FUSED_WAVES;
    const bool valid = t < M;
    const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
    const u32x4 *bp = B_LDS ? nullptr : reinterpret_cast<const u32x4 *>(A.bsrc + (size_t)(valid ? t : 0) * A.ldb + 8 * g);
    const size_t bplane16 = A.bplane / 8;

    for (int item = wg; item < A.n_items; item += nwg) {
        f32x4 acc[TG];
        const u32x4 *wp[TG];
#pragma unroll
        for (int j = 0; j < TG; j++) {
            acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
            wp[j] = A.Wp + ((size_t)(item * TG + j) * KS) * 64 + lane;
        }
        u32x4 wa[U][TG], wb[U][TG], ba[U][2], bb[U][2];

#define FUSED_LOAD(WF, BF, KS_AT)                                                                   \
    _Pragma("unroll") for (int u = 0; u < U; u++) {                                                 \
        const int ksu_ = (KS_AT) + u;                                                               \
        const bool in_ = ksu_ < ks1;                                                                \
        _Pragma("unroll") for (int j = 0; j < TG; j++)                                              \
            WF[u][j] = in_ ? __builtin_nontemporal_load(wp[j] + (size_t)ksu_ * 64) : zero;          \
        if (!B_LDS) {                                                                               \
            BF[u][0] = (in_ && valid) ? bp[(size_t)ksu_ * 4] : zero;                                \
            BF[u][1] = (in_ && valid) ? bp[(size_t)ksu_ * 4 + bplane16] : zero;                     \
        }                                                                                           \
    }
#define FUSED_MMA(WF, BF, KS_AT)                                                                    \
    _Pragma("unroll") for (int u = 0; u < U; u++) {                                                 \
        const int ksu_ = (KS_AT) + u;                                                               \
        u32x4 bh_ = zero, bl_ = zero;                                                               \
        if (B_LDS) {                                                                                \
            if (valid && ksu_ < ks1) {                                                              \
                bh_ = lds_act[((ksu_ * 2 + 0) * 4 + g) * M + t];                                    \
                bl_ = lds_act[((ksu_ * 2 + 1) * 4 + g) * M + t];                                    \
            }                                                                                       \
        } else {                                                                                    \
            bh_ = BF[u][0];                                                                         \
            bl_ = BF[u][1];                                                                         \
        }                                                                                           \
        _Pragma("unroll") for (int j = 0; j < TG; j++) {                                            \
            acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, WF[u][j]),  \
                                                             __builtin_bit_cast(bf16x8, bh_), acc[j], 0, 0, 0); \
            acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, WF[u][j]),  \
                                                             __builtin_bit_cast(bf16x8, bl_), acc[j], 0, 0, 0); \
        }                                                                                           \
    }

        FUSED_LOAD(wa, ba, ks0)
        for (int ks = ks0; ks < ks1; ks += 2 * U) {
            FUSED_LOAD(wb, bb, ks + U)
            FUSED_MMA(wa, ba, ks)
            FUSED_LOAD(wa, ba, ks + 2 * U)
            FUSED_MMA(wb, bb, ks + U)
        }
#undef FUSED_LOAD
#undef FUSED_MMA

        if (item + nwg >= A.n_items) ts_mark(P, TS_LOOP);
        // fixed-order reduction of the 8 K slices through LDS, then one wave per tile applies the epilogue
#pragma unroll
        for (int j = 0; j < TG; j++) red[(w * TG + j) * 64 + lane] = acc[j];
        __syncthreads();
        if (EPI == EPI_SWIGLU) {
            if (w == 0) {                         // TG == 2: tile 0 = gate, tile 1 = up, same 16 features
                f32x4 gsum = red[lane], usum = red[64 + lane];
#pragma unroll
                for (int ww = 1; ww < FUSED_WAVES; ww++) {
                    gsum += red[(ww * TG) * 64 + lane];
                    usum += red[(ww * TG + 1) * 64 + lane];
                }
                if (valid) {
                    float f[4];
#pragma unroll
                    for (int r = 0; r < 4; r++) f[r] = gsum[r] / (1.0f + expf(-gsum[r])) * usum[r];
                    u32x2 hi, lo;
                    split4(f, hi, lo);
                    const __amdgpu_buffer_rsrc_t rf = co_rsrc(P.act, 2 * (P.act_plane * 2));
                    const int off = (int)(((size_t)t * P.F + item * 16 + 4 * g) * 2);
                    co_st64(rf, off, hi);
                    co_st64(rf, off + (int)(P.act_plane * 2), lo);
                }
            }
        } else if (w < TG) {
            f32x4 sum = red[w * 64 + lane];
#pragma unroll
            for (int ww = 1; ww < FUSED_WAVES; ww++) sum += red[(ww * TG + w) * 64 + lane];
            gemm_epilogue<TG, EPI>(P, A, item, w, sum, lane);
        }
        __syncthreads();
    }
}

// Block attention for one 16-row tile per sequence (m <= 16).
template <int DH>
__device__ void phase_attn(const FusedParams &P, int layer, char *smem, int wg, int nwg) {
    constexpr int PS = DH + 4;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int col = lane & 15, g = lane >> 4;
    float *lacc = reinterpret_cast<float *>(smem);              // [8 waves][16 rows][PS]
    __shared__ int s_last;
    const KvGeom geo{P.Bmax, P.H, P.dh, P.seq_pad, P.L, P.kperm};
    const __amdgpu_buffer_rsrc_t ro = co_rsrc(P.act, 2 * (P.act_plane * 2));
    const int items = P.B * P.H * P.kg_max;
    for (int item = wg; item < items; item += nwg) {
        const int kg = item % P.kg_max, hh = (item / P.kg_max) % P.H, b = item / (P.kg_max * P.H);
        const int tlen = P.cache_len[b];
        const int nk = max(0, min(tlen + P.m, P.seq_pad));
        const int n_groups = (nk + 255) / 256;
        if (kg >= n_groups) continue;                            // uniform for the workgroup
        const int kb = (kg * FUSED_WAVES + w) * 32;
        const int qpos = tlen + col;
        f32x4 oacc[DH / 16];
#pragma unroll
        for (int dt = 0; dt < DH / 16; dt++) oacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        float mloc = -INFINITY, lloc = 0.f;
        if (kb < nk) {
            const bf16_t *kc = P.kv + kv_k_off(geo, layer, b, hh);
            const bf16_t *vc = P.kv + kv_v_off(geo, layer, b, hh);
            // issue every load of this 32-key tile up front: q (both planes), K, V
            u32x4 qf[DH / 32][2], kf[2][DH / 32], vf[DH / 16];
#pragma unroll
            for (int s = 0; s < DH / 32; s++) {
                qf[s][0] = qf[s][1] = u32x4{0u, 0u, 0u, 0u};
                if (col < P.m) {
                    const bf16_t *qp = P.q + (size_t)(b * P.m + col) * P.hd + hh * DH + s * 32 + 8 * g;
                    qf[s][0] = *reinterpret_cast<const u32x4 *>(qp);
                    qf[s][1] = *reinterpret_cast<const u32x4 *>(qp + P.q_plane);
                }
            }
#pragma unroll
            for (int T = 0; T < 2; T++) {
                const int key = kb + 8 * (col >> 2) + 4 * T + (col & 3);
#pragma unroll
                for (int s = 0; s < DH / 32; s++)
                    kf[T][s] = *reinterpret_cast<const u32x4 *>(kc + (size_t)key * DH + 8 * g + s * 32);
            }
#pragma unroll
            for (int dt = 0; dt < DH / 16; dt++)
                vf[dt] = *reinterpret_cast<const u32x4 *>(vc + (size_t)(dt * 16 + col) * P.seq_pad + kb + 8 * g);
            f32x4 sT[2];
#pragma unroll
            for (int T = 0; T < 2; T++) {
                sT[T] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < DH / 32; s++) {
                    sT[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[T][s]),
                                                                    __builtin_bit_cast(bf16x8, qf[s][0]), sT[T], 0, 0, 0);
                    sT[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[T][s]),
                                                                    __builtin_bit_cast(bf16x8, qf[s][1]), sT[T], 0, 0, 0);
                }
            }
            float sv[8];
            float mx = -INFINITY;
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const int key = kb + 8 * g + j;
                const float s = sT[j >> 2][j & 3] * P.scale;
                sv[j] = (key <= qpos && key < nk) ? s : -INFINITY;
                mx = fmaxf(mx, sv[j]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            float pv[8];
            float psum = 0.f;
#pragma unroll
            for (int j = 0; j < 8; j++) {
                pv[j] = (sv[j] == -INFINITY) ? 0.f : expf(sv[j] - mx);
                psum += pv[j];
            }
            psum += __shfl_xor(psum, 16, 64);
            psum += __shfl_xor(psum, 32, 64);
            mloc = mx;
            lloc = psum;
            u32x4 pf, pl;
            split8(pv, pf, pl);
            const bool tail = kb + 32 > nk;
#pragma unroll
            for (int dt = 0; dt < DH / 16; dt++) {
                u32x4 vv = vf[dt];
                if (tail) {
#pragma unroll
                    for (int ww = 0; ww < 4; ww++) {
                        const int k0 = kb + 8 * g + 2 * ww;
                        vv[ww] &= (k0 < nk ? 0x0000FFFFu : 0u) | (k0 + 1 < nk ? 0xFFFF0000u : 0u);
                    }
                }
                oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vv),
                                                                   __builtin_bit_cast(bf16x8, pf), oacc[dt], 0, 0, 0);
                oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vv),
                                                                   __builtin_bit_cast(bf16x8, pl), oacc[dt], 0, 0, 0);
            }
        }
        // per-wave state to LDS: row = col, entries dt*16 + 4g + r
        float *lw = lacc + (size_t)(w * 16 + col) * PS;
#pragma unroll
        for (int dt = 0; dt < DH / 16; dt++) *reinterpret_cast<f32x4 *>(lw + dt * 16 + 4 * g) = oacc[dt];
        if (g == 0) {
            lw[DH] = mloc;
            lw[DH + 1] = lloc;
        }
        __syncthreads();
        // merge the 8 waves: thread -> (row, 4 consecutive outputs); partial state goes out coherently
        const size_t part_elems = (size_t)16 * PS;
        const __amdgpu_buffer_rsrc_t rp =
            co_rsrc(P.attn_part + (size_t)((b * P.H + hh) * P.kg_max) * part_elems, sizeof(float) * part_elems * P.kg_max);
        for (int idx = tid; idx < 16 * (DH / 4); idx += FUSED_THREADS) {
            const int r = idx / (DH / 4), x4 = idx % (DH / 4);
            float mstar = -INFINITY;
#pragma unroll
            for (int ww = 0; ww < FUSED_WAVES; ww++) mstar = fmaxf(mstar, lacc[(size_t)(ww * 16 + r) * PS + DH]);
            f32x4 num = f32x4{0.f, 0.f, 0.f, 0.f};
            float den = 0.f;
#pragma unroll
            for (int ww = 0; ww < FUSED_WAVES; ww++) {
                const float *src = lacc + (size_t)(ww * 16 + r) * PS;
                const float mw = src[DH];
                const float wgt = (mw == -INFINITY) ? 0.f : expf(mw - mstar);
                num += *reinterpret_cast<const f32x4 *>(src + x4 * 4) * wgt;
                den += src[DH + 1] * wgt;
            }
            const int off = (int)(((size_t)kg * part_elems + (size_t)r * PS + x4 * 4) * 4);
            co_st128f(rp, off, num);
            if (x4 == 0) {
                co_st32f(rp, (int)(((size_t)kg * part_elems + (size_t)r * PS + DH) * 4), mstar);
                co_st32f(rp, (int)(((size_t)kg * part_elems + (size_t)r * PS + DH + 1) * 4), den);
            }
        }
        __syncthreads();        // every partial store of this workgroup has been acknowledged
        if (tid == 0) {
            const unsigned old = __hip_atomic_fetch_add(P.attn_cnt + b * P.H + hh, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = (old == (unsigned)(n_groups - 1));
        }
        __syncthreads();
        if (s_last) {           // the last key group to finish merges all of them
            for (int idx = tid; idx < P.m * (DH / 4); idx += FUSED_THREADS) {
                const int r = idx / (DH / 4), x4 = idx % (DH / 4);
                float mstar = -INFINITY;
                for (int c = 0; c < n_groups; c++)
                    mstar = fmaxf(mstar, co_ld32f(rp, (int)(((size_t)c * part_elems + (size_t)r * PS + DH) * 4)));
                f32x4 num = f32x4{0.f, 0.f, 0.f, 0.f};
                float den = 0.f;
                for (int c = 0; c < n_groups; c++) {
                    const int base = (int)(((size_t)c * part_elems + (size_t)r * PS) * 4);
                    const float mc = co_ld32f(rp, base + DH * 4);
                    const float wgt = (mc == -INFINITY) ? 0.f : expf(mc - mstar);
                    num += co_ld128f(rp, base + x4 * 16) * wgt;
                    den += co_ld32f(rp, base + (DH + 1) * 4) * wgt;
                }
                const float inv = den > 0.f ? 1.0f / den : 0.f;
                float o[4] = {num[0] * inv, num[1] * inv, num[2] * inv, num[3] * inv};
                u32x2 hi, lo;
                split4(o, hi, lo);
                const int off = (int)(((size_t)(b * P.m + r) * P.hd + hh * DH + x4 * 4) * 2);
                co_st64(ro, off, hi);
                co_st64(ro, off + (int)(P.act_plane * 2), lo);
            }
            if (tid == 0) __hip_atomic_store(P.attn_cnt + b * P.H + hh, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
    }
}

__device__ void phase_trace(const FusedParams &P, int slot, int wg, int nwg) {
    const size_t n = (size_t)P.M * P.d;
    for (size_t i = (size_t)wg * FUSED_THREADS + threadIdx.x; i < n; i += (size_t)nwg * FUSED_THREADS)
        P.trace[(size_t)slot * n + i] = P.h[i];
}

template <int DH>
__device__ void run_phase(const FusedParams &P, int phase, int layer, char *smem, int wg, int nwg) {
    GemmArgs A;
    A.layer = layer;
    A.gain = nullptr;
    A.bsrc = nullptr;
    A.bplane = 0;
    A.ldb = 0;
    if (phase == PH_EMBED) {
        phase_embed(P, wg, nwg);
    } else if (phase == PH_QKV) {
        const FusedLayer lw = P.layers[layer];
        A.Wp = lw.qkv;
        A.KS = P.d / 32;
        A.gain = lw.attn_norm;
        A.n_items = (3 * P.hd / 16) / P.tg_qkv;
        if (P.tg_qkv == 3)
            gemm_phase<3, EPI_QKV, true, 2>(P, A, smem, wg, nwg);
        else
            gemm_phase<1, EPI_QKV, true, 8>(P, A, smem, wg, nwg);
    } else if (phase == PH_ATTN) {
        phase_attn<DH>(P, layer, smem, wg, nwg);
    } else if (phase == PH_O) {
        const FusedLayer lw = P.layers[layer];
        A.Wp = lw.o;
        A.KS = P.hd / 32;
        A.n_items = P.d / 16;
        A.bsrc = P.act;
        A.bplane = P.act_plane;
        A.ldb = P.hd;
        gemm_phase<1, EPI_RESID, false, 4>(P, A, smem, wg, nwg);
    } else if (phase == PH_GU) {
        const FusedLayer lw = P.layers[layer];
        A.Wp = lw.gu;
        A.KS = P.d / 32;
        A.gain = lw.ffn_norm;
        A.n_items = P.F / 16;
        gemm_phase<2, EPI_SWIGLU, true, 4>(P, A, smem, wg, nwg);
    } else if (phase == PH_DOWN) {
        const FusedLayer lw = P.layers[layer];
        A.Wp = lw.down;
        A.KS = P.F / 32;
        A.n_items = P.d / 16;
        A.bsrc = P.act;
        A.bplane = P.act_plane;
        A.ldb = P.F;
        gemm_phase<1, EPI_RESID, false, 4>(P, A, smem, wg, nwg);
    } else if (phase == PH_LM) {
        A.Wp = P.lm;
        A.KS = P.d / 32;
        A.gain = P.final_norm;
        A.n_items = (P.V / 16) / P.tg_lm;
        if (P.tg_lm == 2)
            gemm_phase<2, EPI_LOGITS, true, 4>(P, A, smem, wg, nwg);
        else
            gemm_phase<1, EPI_LOGITS, true, 8>(P, A, smem, wg, nwg);
    } else if (phase == PH_TRACE) {
        phase_trace(P, layer, wg, nwg);
    }
}

// one launch per phase
template <int DH>
__global__ __launch_bounds__(FUSED_THREADS, 1) void k_fused_phase(FusedParams P, int phase, int layer) {
    extern __shared__ __align__(16) char smem[];
    run_phase<DH>(P, phase, layer, smem, blockIdx.x, gridDim.x);
}

// the whole forward in one launch
template <int DH>
__global__ __launch_bounds__(FUSED_THREADS, 1) void k_verify_persistent(FusedParams P) {
    extern __shared__ __align__(16) char smem[];
    const int wg = blockIdx.x, nwg = gridDim.x;
    unsigned long long epoch = P.bar_base;   // device-wide barriers completed before this launch
    P.ts_slot = 0;
#define FUSED_STEP(PHASE, LAYER)                      \
    ts_mark(P, TS_START);                             \
    run_phase<DH>(P, PHASE, LAYER, smem, wg, nwg);    \
    ts_mark(P, TS_EPILOGUE);                          \
    grid_barrier(P, ++epoch);                         \
    ts_mark(P, TS_BARRIER);                           \
    P.ts_slot += TS_PER_PHASE;
    FUSED_STEP(PH_EMBED, 0)
    if (P.trace) run_phase<DH>(P, PH_TRACE, 0, smem, wg, nwg);
    for (int l = 0; l < P.L; l++) {
        FUSED_STEP(PH_QKV, l)
        FUSED_STEP(PH_ATTN, l)
        FUSED_STEP(PH_O, l)
        FUSED_STEP(PH_GU, l)
        FUSED_STEP(PH_DOWN, l)
        if (P.trace) run_phase<DH>(P, PH_TRACE, l + 1, smem, wg, nwg);
    }
#undef FUSED_STEP
    ts_mark(P, TS_START);
    run_phase<DH>(P, PH_LM, 0, smem, wg, nwg);
    ts_mark(P, TS_EPILOGUE);
}

// ------------------------------------------------------------------------------- host side

struct FusedState {
    FusedLayer *layers = nullptr;
    float *cs = nullptr;
    unsigned *attn_cnt = nullptr;
    unsigned long long *bar = nullptr;
    unsigned *err = nullptr;
    unsigned long long bar_epoch = 0;
    int grid = 0, kg_max = 0, tg_qkv = 1, tg_lm = 1;
    size_t lds_bytes = 0;
    int lds_red_off = 0, lds_rstd_off = 0;
    int m_limit = 0;
    int mode = 2;      // 0: off, 1: one launch per phase, 2: persistent
};

static int32_t fused_alloc(csd_model *mod, void **p, size_t bytes, bool zero, hipStream_t st) {
    CSD_HIP(hipMalloc(p, bytes));
    mod->allocs.push_back(*p);
    if (zero) CSD_HIP(hipMemsetAsync(*p, 0, bytes, st));
    return CSD_OK;
}

int32_t csd_fused_init(csd_model *mod, hipStream_t st) {
    const csd_model_cfg &c = mod->cfg;
    mod->fused = nullptr;
    if (!mod->mfma || !mod->mfma_attn) return CSD_OK;
    const char *e = getenv("CSD_PATH");
    int mode = 2;
    if (e && strcmp(e, "multikernel") == 0) mode = 0;
    if (e && strcmp(e, "phases") == 0) mode = 1;
    if (mode == 0) return CSD_OK;
    int dev = 0, cus = 0, lds_max = 0;
    CSD_HIP(hipGetDevice(&dev));
    CSD_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    CSD_HIP(hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
    const int d = c.d_model, hd = mod->hd, F = c.d_ffn, V = c.vocab, dh = c.head_dim;
    // rows the LDS-resident activations allow: M*d*4 bytes + reduction scratch + attention merge area
    const int red_bytes = FUSED_WAVES * 3 * 64 * 16;
    const int attn_bytes = FUSED_WAVES * 16 * (dh + 4) * 4;
    int m_limit = 16;
    while (m_limit > 0 && (size_t)m_limit * d * 4 + red_bytes + 256 > (size_t)lds_max) m_limit--;
    if (m_limit < 1 || attn_bytes > lds_max) return CSD_OK;
    if (d % 32 || hd % 32 || F % 32 || V % 16 || (F / 16) < 1) return CSD_OK;
    FusedState *fs = new FusedState();
    fs->mode = mode;
    fs->m_limit = m_limit < mod->m_max ? m_limit : mod->m_max;
    const int m_cap = fs->m_limit;
    size_t act_bytes = (size_t)m_cap * d * 4;
    fs->lds_red_off = (int)((act_bytes + 255) / 256 * 256);
    fs->lds_rstd_off = fs->lds_red_off + red_bytes;
    fs->lds_bytes = (size_t)fs->lds_rstd_off + 256;
    if (fs->lds_bytes < (size_t)attn_bytes) fs->lds_bytes = attn_bytes;
    fs->grid = cus;
    fs->kg_max = (mod->seq_pad + 255) / 256;
    fs->tg_qkv = ((3 * hd / 16) / 3 >= cus) ? 3 : 1;
    fs->tg_lm = ((V / 16) % 2 == 0) ? 2 : 1;
    int32_t rc;
    std::vector<FusedLayer> hl(c.n_layers);
    for (int l = 0; l < c.n_layers; l++) {
        const LayerW &lw = mod->layers[l];
        hl[l] = FusedLayer{(const u32x4 *)lw.qkv.data, (const u32x4 *)lw.o.data, (const u32x4 *)lw.gu.data,
                           (const u32x4 *)lw.down.data, lw.attn_norm, lw.ffn_norm};
    }
    if ((rc = fused_alloc(mod, (void **)&fs->layers, sizeof(FusedLayer) * c.n_layers, false, st)) != CSD_OK) return rc;
    CSD_HIP(hipMemcpy(fs->layers, hl.data(), sizeof(FusedLayer) * c.n_layers, hipMemcpyHostToDevice));
    if ((rc = fused_alloc(mod, (void **)&fs->cs, sizeof(float) * 16 * dh, false, st)) != CSD_OK) return rc;
    if ((rc = fused_alloc(mod, (void **)&fs->attn_cnt, sizeof(unsigned) * c.max_batch * c.n_heads, true, st)) != CSD_OK) return rc;
    if ((rc = fused_alloc(mod, (void **)&fs->bar, 8 * BAR_STRIDE * 64, true, st)) != CSD_OK) return rc;
    if ((rc = fused_alloc(mod, (void **)&fs->err, 256, true, st)) != CSD_OK) return rc;
    // attention partials: [Bmax][H][kg_max][16][dh+4]; reuse the model's buffer when large enough
    const size_t need = sizeof(float) * (size_t)c.max_batch * c.n_heads * fs->kg_max * 16 * (dh + 4);
    if ((rc = fused_alloc(mod, (void **)&mod->fused_attn_part, need, false, st)) != CSD_OK) return rc;
    if (dh == 128) {
        CSD_HIP(hipFuncSetAttribute((const void *)k_verify_persistent<128>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)fs->lds_bytes));
        CSD_HIP(hipFuncSetAttribute((const void *)k_fused_phase<128>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)fs->lds_bytes));
    } else {
        CSD_HIP(hipFuncSetAttribute((const void *)k_verify_persistent<64>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)fs->lds_bytes));
        CSD_HIP(hipFuncSetAttribute((const void *)k_fused_phase<64>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)fs->lds_bytes));
    }
    mod->fused = fs;
    return CSD_OK;
}

void csd_fused_free(csd_model *mod) {
    delete (FusedState *)mod->fused;
    mod->fused = nullptr;
}

bool csd_fused_eligible(const csd_model *mod, int32_t B, int32_t m) {
    const FusedState *fs = (const FusedState *)mod->fused;
    return fs && B * m <= fs->m_limit && B * m <= 16 && m <= 16;
}

int32_t csd_fused_path(const csd_model *mod, int32_t B, int32_t m) {
    const FusedState *fs = (const FusedState *)mod->fused;
    return csd_fused_eligible(mod, B, m) ? fs->mode : 0;
}

int32_t csd_fused_error(const csd_model *mod, uint32_t *flag) {
    const FusedState *fs = (const FusedState *)mod->fused;
    *flag = 0;
    if (!fs) return CSD_OK;
    CSD_HIP(hipMemcpy(flag, fs->err, sizeof(uint32_t), hipMemcpyDeviceToHost));
    return CSD_OK;
}

int32_t csd_fused_enqueue(csd_model *mod, void *kv, const int32_t *tokens, const int32_t *cache_len, int32_t B,
                          int32_t m, float *logits, hipStream_t st) {
    FusedState *fs = (FusedState *)mod->fused;
    const csd_model_cfg &c = mod->cfg;
    FusedParams P;
    P.M = B * m;
    P.m = m;
    P.B = B;
    P.d = c.d_model;
    P.hd = mod->hd;
    P.H = c.n_heads;
    P.dh = c.head_dim;
    P.F = c.d_ffn;
    P.V = c.vocab;
    P.L = c.n_layers;
    P.seq_pad = mod->seq_pad;
    P.Bmax = c.max_batch;
    P.kperm = mod->kperm ? 1 : 0;
    P.kg_max = fs->kg_max;
    P.tg_qkv = fs->tg_qkv;
    P.tg_lm = fs->tg_lm;
    P.lds_red_off = fs->lds_red_off;
    P.lds_rstd_off = fs->lds_rstd_off;
    P.eps = c.rms_eps;
    P.scale = 1.0f / sqrtf((float)c.head_dim);
    P.theta = c.rope_theta;
    P.tokens = tokens;
    P.cache_len = cache_len;
    P.embed = (const bf16_t *)mod->embed;
    P.layers = fs->layers;
    P.final_norm = mod->final_norm;
    P.lm = (const u32x4 *)mod->lm.data;
    P.h = mod->h;
    P.q = (bf16_t *)mod->qbuf;
    P.q_plane = mod->q_plane;
    P.act = (bf16_t *)mod->act;
    P.act_plane = mod->act_plane;
    P.cs = fs->cs;
    P.kv = (bf16_t *)kv;
    P.attn_part = mod->fused_attn_part;
    P.attn_cnt = fs->attn_cnt;
    P.logits = logits;
    P.bar = fs->bar;
    P.err = fs->err;
    P.trace = mod->trace;
    P.ts = (unsigned long long *)mod->fused_ts;
    P.ts_slot = 0;
    const dim3 grid(fs->grid), block(FUSED_THREADS);
    if (fs->mode == 2) {
        P.bar_base = fs->bar_epoch;
        fs->bar_epoch += (unsigned long long)(1 + 5 * c.n_layers);
        ProfScope ps(mod, st, CSD_PROF_GEMM);
        if (c.head_dim == 128)
            hipLaunchKernelGGL((k_verify_persistent<128>), grid, block, fs->lds_bytes, st, P);
        else
            hipLaunchKernelGGL((k_verify_persistent<64>), grid, block, fs->lds_bytes, st, P);
        CSD_LAUNCH_CHECK();
        return CSD_OK;
    }
    P.bar_base = 0;
    auto launch = [&](int phase, int layer, int cls) -> int32_t {
        ProfScope ps(mod, st, cls);
        if (c.head_dim == 128)
            hipLaunchKernelGGL((k_fused_phase<128>), grid, block, fs->lds_bytes, st, P, phase, layer);
        else
            hipLaunchKernelGGL((k_fused_phase<64>), grid, block, fs->lds_bytes, st, P, phase, layer);
        CSD_LAUNCH_CHECK();
        return CSD_OK;
    };
    int32_t rc;
    if ((rc = launch(PH_EMBED, 0, CSD_PROF_OTHER)) != CSD_OK) return rc;
    if (P.trace && (rc = launch(PH_TRACE, 0, CSD_PROF_OTHER)) != CSD_OK) return rc;
    for (int l = 0; l < c.n_layers; l++) {
        if ((rc = launch(PH_QKV, l, CSD_PROF_GEMM)) != CSD_OK) return rc;
        if ((rc = launch(PH_ATTN, l, CSD_PROF_ATTN)) != CSD_OK) return rc;
        if ((rc = launch(PH_O, l, CSD_PROF_GEMM)) != CSD_OK) return rc;
        if ((rc = launch(PH_GU, l, CSD_PROF_GEMM)) != CSD_OK) return rc;
        if ((rc = launch(PH_DOWN, l, CSD_PROF_GEMM)) != CSD_OK) return rc;
        if (P.trace && (rc = launch(PH_TRACE, l + 1, CSD_PROF_OTHER)) != CSD_OK) return rc;
    }
    return launch(PH_LM, 0, CSD_PROF_GEMM);
}
