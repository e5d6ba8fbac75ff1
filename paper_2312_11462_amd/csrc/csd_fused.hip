// Single-launch review forward for small blocks (M = B*m <= 16 rows) of the LLaMA-style decoder: one
// persistent grid, one workgroup of 8 waves per compute unit, walks through every phase of every layer
// with a device-wide barrier between phases, so the weights stream from HBM without kernel boundaries
// in between.
//
// Phases of a layer (five barriers):
//   1. QKV projection; epilogue: scale by the row's RMS factor, rotate q and k (the projection's
//      output features are tiled in rotary pair order, so a 16-feature MFMA tile holds whole pairs),
//      append K and V to the cache, store q.
//   2. Block attention over the cached prefix: a workgroup takes (sequence, head, 256 keys), its 8
//      waves one 32-key tile each; partial softmax states merge in LDS, then across workgroups by
//      the last one to arrive.
//   3. Output projection; epilogue h += , and the next GEMM's input h*gain as two bf16 planes.
//   4. Gate/up projection; epilogue f = silu(gate) * up (after the RMS factor).
//   5. Down projection; epilogue as in 3.
// RMSNorm is folded around the GEMM: rmsnorm(h)*g @ W = rstd(row) * ((h*g) @ W), so the producer of h
// writes h*g (two bf16 planes) plus per-tile sums of squares, and the consumer multiplies its output
// rows by rstd = 1/sqrt(sum/d + eps).  No phase needs a normalisation pass over the activations.
// A GEMM work item is a group of TG adjacent 16-feature tiles over the whole K.  Wave 0 of a workgroup
// is its service wave (barrier, row scales, reduction and epilogue of each item); waves 1-7 split K,
// stream their weight fragments through a register ring that runs ahead across items and across the
// barrier, multiply them with the activation fragments (copied into LDS once per phase, or read from
// L2 through a second ring where they do not fit), and hand their partial sums to the service wave
// through LDS, which adds them in a fixed order (deterministic).  No partial sum travels through HBM.
//
// Data one workgroup writes for another goes out with write-through stores; every exchanged buffer has
// one instance per producing phase, so consumers read with ordinary cached loads and no cache has to be
// invalidated after a barrier.  The barrier itself is a set of one-byte flags in uncached memory, polled
// with scalar loads.
//
// The same phase functions are also launchable one kernel per phase (debugging / comparison).
// Tuning and test knobs read from the environment at csd_model_create: CSD_PATH=multikernel|phases,
// CSD_FUSED_PF (ring slots prefetched across a barrier), CSD_FUSED_FRESH=0 (reuse the exchange buffers
// and invalidate L2 after every barrier), CSD_FUSED_ARRIVE_FIRST=0, CSD_FUSED_VECTOR_POLL,
// CSD_FUSED_M_LDS (cap on the rows kept in LDS), CSD_FUSED_L2B (enables the variant that reads the
// activation fragments from L2, for blocks of up to 16 rows that do not fit LDS).
#include <mutex>
#include <vector>

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
    int arrive_first;  // 1: streaming waves hold their prefetch until the service wave has signalled the barrier
    int bar_scalar;    // 1: the barrier flags live in uncached memory and are polled with scalar loads
    int fresh;         // 1: every phase writes its own instance of the exchange buffers (no L2 invalidate)
    int pf;            // ring slots of the next phase's weights issued before the barrier wait
    int lds_red_off, lds_rstd_off;   // LDS: [0, red_off) activation fragments (or the attention merge area),
                                     // then the split-K reduction scratch, then 16 floats of rstd
    float eps, scale, theta;
    const int32_t *tokens, *cache_len;
    const bf16_t *embed;
    const FusedLayer *layers;
    const float *final_norm;
    const u32x4 *lm;
    // Exchange buffers, one instance per producing phase of the whole forward (never reused inside a
    // launch): xh/xhg/xssq have 2L+1 slots (embedding, then after the output and the down projection of
    // every layer), xq/xattn/xffn one per layer.  All hold 16 rows.
    float *xh;         // residual stream, fp32 [slot][16][d]
    bf16_t *xhg;       // h * gain of the next norm, two bf16 planes [slot][2][16][d]: input of QKV / gate-up / LM head
    float *xssq;       // [slot][16 rows][d/16 tiles] sums of squares of h, per tile
    bf16_t *xq;        // rotated queries, two planes [layer][2][16][hd]
    bf16_t *xattn;     // attention output, two planes [layer][2][16][hd]
    bf16_t *xffn;      // SwiGLU output, two planes [layer][2][16][F]
    size_t q_plane, hg_plane, ffn_plane;      // elements between the two planes (16 rows)
    float *cs;         // rotary table [M][dh/2][cos, sin]
    bf16_t *kv;
    float *attn_part;
    unsigned *attn_cnt;
    float *logits;
    unsigned char *bar;       // barrier flags: BAR_REPLICAS copies of one byte per workgroup
    unsigned bar_base;
    unsigned *err;
    float *trace;
    unsigned long long *ts;   // optional timing marks [mark][workgroup] (100 MHz wall clock), see TS_*
};

enum { TS_START = 0, TS_PROLOGUE = 1, TS_LOOP = 2, TS_EPILOGUE = 3, TS_BARRIER = 4, TS_PER_PHASE = 5 };
// Device code takes the launch parameters by reference to the kernel argument and never writes to
// them.  (Attempts to keep them wholly in scalar registers, by inlining every phase or by reading the
// kernel-argument segment directly, made the register allocator spill thousands of vector registers
// in the single-launch kernel; with the three small phases left as real calls it spills none.)
typedef const FusedParams CParams;

// What changes from phase to phase: the instances of the exchange buffers the phase reads and writes,
// and where its timing marks go.  Kept apart from FusedParams, which stays a read-only kernel argument
// (anything mutable in it would move the whole structure into scratch memory, and scratch accesses
// queue behind the weight stream like every other vector memory access).
struct PhaseBufs {
    const float *h_in;
    float *h_out;
    const bf16_t *hg_in;
    bf16_t *hg_out;
    const float *ssq_in;
    float *ssq_out;
    bf16_t *q, *attn_o, *ffn_a;
    int ts_slot;              // first mark index of the phase
};

__device__ __forceinline__ void ts_mark(CParams &P, const PhaseBufs &X, int which) {
    if (P.ts && threadIdx.x == 0) P.ts[(size_t)(X.ts_slot + which) * gridDim.x + blockIdx.x] = wall_clock64();
}

// A buffer instance is written in exactly one phase and read only in later phases; with P.fresh every
// phase of the forward has its own, so no cache ever holds a stale line of it during the launch.
__device__ __forceinline__ PhaseBufs make_bufs(CParams &P, int phase, int layer, int ts_slot) {
    PhaseBufs X;
    X.ts_slot = ts_slot;
    if (!P.fresh) {       // one instance of each buffer, reused by every layer (the barrier then invalidates L2)
        X.h_in = X.h_out = P.xh;
        X.hg_in = X.hg_out = P.xhg;
        X.ssq_in = X.ssq_out = P.xssq;
        X.q = P.xq;
        X.attn_o = P.xattn;
        X.ffn_a = P.xffn;
        return X;
    }
    // slot of the residual stream entering the phase: 2l for the attention half, 2l+1 for the FFN half
    const int s_in = phase == PH_EMBED ? 0 : phase == PH_LM ? 2 * P.L : (phase == PH_GU || phase == PH_DOWN) ? 2 * layer + 1 : 2 * layer;
    const int s_out = phase == PH_EMBED ? 0 : s_in + 1;
    const size_t hs = (size_t)16 * P.d;
    X.h_in = P.xh + hs * s_in;
    X.h_out = P.xh + hs * s_out;
    X.hg_in = P.xhg + 2 * hs * s_in;
    X.hg_out = P.xhg + 2 * hs * s_out;
    X.ssq_in = P.xssq + (size_t)(P.d / 16) * 16 * s_in;
    X.ssq_out = P.xssq + (size_t)(P.d / 16) * 16 * s_out;
    X.q = P.xq + (size_t)2 * 16 * P.hd * layer;
    X.attn_o = P.xattn + (size_t)2 * 16 * P.hd * layer;
    X.ffn_a = P.xffn + (size_t)2 * 16 * P.F * layer;
    return X;
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

// Workgroup barrier after which every global store issued before it by any wave of the workgroup has
// been acknowledged.  The compiler's workgroup barrier alone does not give that: waves of a workgroup
// share one vector cache, so it only waits for LDS traffic, while the write-through stores here must have
// reached the level other workgroups read from before anything (a counter, a flag) announces them.
__device__ __forceinline__ void stores_acked_sync() {
    __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0)
    __syncthreads();
}

// ------------------------------------------------------------------------------ grid barrier

// Flag barrier without read-modify-write atomics: workgroup w records the barrier it has reached in its
// one-byte flag, and the service wave of every workgroup polls all flags with one
// 4-byte load per lane (4 flags each, up to 256 workgroups).  Polling is what loads the memory
// channel that holds the flags, and the weight stream needs every channel, so the flags exist in
// BAR_REPLICAS copies on different channels: an arriving workgroup writes all copies (one store
// instruction, one lane per copy) and polls only copy (workgroup index mod BAR_REPLICAS).
// Barrier numbers only grow (the host passes the number completed by earlier launches).  While a
// workgroup waits for barrier e, another can be one barrier behind (not arrived: e - 1) or one ahead (it
// saw everyone arrive, had no work in the next phase and has already arrived at e + 1), never more.  A
// flag therefore holds its barrier number modulo 4 as one of four bits, 1 << (e % 4), and "everyone has
// arrived at e" is "no flag has the bit of e - 1", a test on the OR of all flags that a faster
// workgroup's next arrival cannot invalidate.  (Waiting for every flag to equal e would miss that
// state for good once a flag has moved on to e + 1.)  Flags of workgroups that do not exist stay 0; the
// flags of those that do start at the bit of barrier 0.
// The wait is bounded: when it gives up it raises the error flag, which also releases every later
// wait, so each wave still exits.
// No cache maintenance is needed here: everything read after a barrier lives in a buffer instance that
// was never read before in this launch (see make_bufs), and the flags themselves are polled with
// loads that bypass the non-coherent caches.
#define BAR_MAX_WG 256
#define BAR_REPLICAS 8
#define BAR_REPLICA_STRIDE (4096 + 256)   /* bytes */
#define BAR_BYTES (BAR_REPLICAS * BAR_REPLICA_STRIDE)

// service_only: only the service wave (wave 0) stored to global memory in this phase (GEMM phases: the
// other waves hand their partial sums over through LDS), so only it waits for its store acknowledgements
// and the streaming waves run straight on to prefetch the next phase's weights.
__device__ __forceinline__ void grid_arrive(CParams &P, unsigned epoch, bool service_only) {
    if (service_only) {
        if (threadIdx.x < 64) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's stores are acknowledged
    } else {
        stores_acked_sync();
    }
    if (threadIdx.x < BAR_REPLICAS) {
        const __amdgpu_buffer_rsrc_t rb = co_rsrc(P.bar, BAR_BYTES);
        __builtin_amdgcn_raw_buffer_store_b8((unsigned char)(1u << (epoch & 3u)), rb, (int)(threadIdx.x * BAR_REPLICA_STRIDE + blockIdx.x), 0,
                                             CSD_SC1);
    }
}

// Between arrive and wait a wave may issue loads that do not depend on other workgroups (the next
// phase's weights); the closing workgroup barrier orders LDS only, so those loads stay in flight.
typedef unsigned u32x16 __attribute__((ext_vector_type(16)));

// Does no flag of replica `fp` (64 dwords of 4 one-byte flags) have a bit of `pat_prev` set?
// Read with scalar loads that bypass the scalar cache (glc): they do not go through the vector memory
// pipeline, so they never queue behind the weight prefetch the compute unit has in flight.  The flag
// memory is allocated uncached, so the loads reach memory whichever L2 serves them.
__device__ __forceinline__ bool flags_clear_scalar(const unsigned char *fp_any, unsigned pat_prev) {
    // the address is the same in every lane, but the compiler may hold it in vector registers
    const unsigned long long a64 = (unsigned long long)fp_any;
    const unsigned lo32 = __builtin_amdgcn_readfirstlane((unsigned)a64);
    const unsigned hi32 = __builtin_amdgcn_readfirstlane((unsigned)(a64 >> 32));
    const unsigned char *fp = reinterpret_cast<const unsigned char *>(((unsigned long long)hi32 << 32) | lo32);
    pat_prev = __builtin_amdgcn_readfirstlane(pat_prev);
    u32x16 a, b, c, d;
    asm volatile("s_load_dwordx16 %0, %4, 0x0 glc\n\t"
                 "s_load_dwordx16 %1, %4, 0x40 glc\n\t"
                 "s_load_dwordx16 %2, %4, 0x80 glc\n\t"
                 "s_load_dwordx16 %3, %4, 0xc0 glc\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&s"(a), "=&s"(b), "=&s"(c), "=&s"(d)
                 : "s"(fp)
                 : "memory");
    const u32x16 o = (a | b) | (c | d);
    unsigned any = 0;
#pragma unroll
    for (int i = 0; i < 16; i++) any |= o[i];
    return (any & pat_prev) == 0u;
}

__device__ __forceinline__ void grid_wait(CParams &P, unsigned epoch) {
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        const __amdgpu_buffer_rsrc_t rb = co_rsrc(P.bar, BAR_BYTES);
        const int rep = (int)((blockIdx.x % BAR_REPLICAS) * BAR_REPLICA_STRIDE);
        const int off = rep + lane * 4;
        const bool scalar = P.bar_scalar != 0;
        const unsigned pat_prev = (1u << ((epoch - 1u) & 3u)) * 0x01010101u;
        unsigned spins = 0;
        bool give_up = __hip_atomic_load(P.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
        while (!give_up) {
            if (scalar) {
                if (flags_clear_scalar(P.bar + rep, pat_prev)) break;
            } else {
                const unsigned f = __builtin_amdgcn_raw_buffer_load_b32(rb, off, 0, CSD_SC1);
                if (__all((f & pat_prev) == 0u)) break;
            }
            ++spins;
            if ((spins & 1023u) == 0u && __hip_atomic_load(P.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)
                give_up = true;
            if (spins > (1u << 20)) {
                if (lane == 0) __hip_atomic_store(P.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                give_up = true;
            }
        }
    }
    // with reused exchange buffers this XCD's L2 may hold the previous layer's lines: drop them
    if (!P.fresh && threadIdx.x == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    lds_sync();
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

// Residual-stream tile hand-over used by the embedding and by the residual epilogues: lane (t, g) holds
// 4 consecutive features of row t of 16-feature tile T.  Writes h, the next GEMM's input h*gain as two
// bf16 planes, and the tile's sum of squares per row.
__device__ __forceinline__ void publish_h_tile(CParams &P, const PhaseBufs &X, const float *__restrict__ gain, int T, int t, int g,
                                               f32x4 hv, bool valid) {
    const __amdgpu_buffer_rsrc_t rh = co_rsrc(X.h_out, sizeof(float) * (size_t)P.M * P.d);
    const __amdgpu_buffer_rsrc_t rg = co_rsrc(X.hg_out, 2 * (P.hg_plane * 2));
    const __amdgpu_buffer_rsrc_t rs = co_rsrc(X.ssq_out, sizeof(float) * (size_t)(P.d / 16) * 16);
    float ss = hv[0] * hv[0] + hv[1] * hv[1] + hv[2] * hv[2] + hv[3] * hv[3];
    ss += __shfl_xor(ss, 16, 64);
    ss += __shfl_xor(ss, 32, 64);
    if (!valid) return;
    const int col = T * 16 + 4 * g;
    const f32x4 gv = *reinterpret_cast<const f32x4 *>(gain + col);
    co_st128f(rh, (int)(((size_t)t * P.d + col) * 4), hv);
    float v[4] = {hv[0] * gv[0], hv[1] * gv[1], hv[2] * gv[2], hv[3] * gv[3]};
    u32x2 hi, lo;
    split4(v, hi, lo);
    const int off = (int)(((size_t)t * P.d + col) * 2);
    co_st64(rg, off, hi);
    co_st64(rg, off + (int)(P.hg_plane * 2), lo);
    if (g == 0) co_st32f(rs, (int)(((size_t)t * (P.d / 16) + T) * 4), ss);
}

// h[r] = E[token[r]] (published as above for the first QKV) and the rotary table of this call's positions
__device__ __noinline__ void phase_embed(CParams &P, int wg, int nwg) {
    const PhaseBufs X = make_bufs(P, PH_EMBED, 0, 0);
    const int lane = threadIdx.x & 63, t = lane & 15, g = lane >> 4;
    const int gw = wg * FUSED_WAVES + (threadIdx.x >> 6), nw = nwg * FUSED_WAVES;
    const bool valid = t < P.M;
    const int tok = valid ? P.tokens[t] : -1;
    for (int T = gw; T < P.d / 16; T += nw) {         // one wave per 16-feature tile, all rows
        f32x4 hv = f32x4{0.f, 0.f, 0.f, 0.f};
        if (tok >= 0 && tok < P.V) {
            const u32x2 e = *reinterpret_cast<const u32x2 *>(P.embed + (size_t)tok * P.d + T * 16 + 4 * g);
            hv = f32x4{__uint_as_float(e[0] << 16), __uint_as_float(e[0] & 0xFFFF0000u), __uint_as_float(e[1] << 16),
                       __uint_as_float(e[1] & 0xFFFF0000u)};
        }
        publish_h_tile(P, X, P.layers[0].attn_norm, T, t, g, hv, valid);
    }
    const __amdgpu_buffer_rsrc_t rc = co_rsrc(P.cs, sizeof(float) * (size_t)P.M * P.dh);
    const size_t gtid = (size_t)wg * FUSED_THREADS + threadIdx.x, gsz = (size_t)nwg * FUSED_THREADS;
    const int half = P.dh / 2;
    for (size_t c = gtid; c < (size_t)P.M * half; c += gsz) {
        const int r = (int)(c / half), x = (int)(c % half);
        const int pos = P.cache_len[r / P.m] + r % P.m;
        const double ang = (double)pos * pow((double)P.theta, -2.0 * (double)x / (double)P.dh);
        co_st32f(rc, (int)(c * 8), (float)cos(ang));
        co_st32f(rc, (int)(c * 8 + 4), (float)sin(ang));
    }
}

struct GemmArgs {
    const u32x4 *Wp;       // tiles [n_tiles][KS][64]
    int KS, n_items;       // k-steps of 32; work items (groups of TG tiles)
    const bf16_t *bsrc;    // B operand rows [M][ldb] in global memory, two planes
    size_t bplane;
    int ldb;
    bool scaled;           // the input is h*gain: multiply output rows by rstd
    const float *next_gain;   // residual epilogue: gain of the norm that follows
    int layer;
};

template <int TG, int EPI>
__device__ __forceinline__ void gemm_epilogue(CParams &P, const PhaseBufs &X, const GemmArgs &A, int item, int j, f32x4 v, int lane,
                                              f32x4 hcur) {
    const int t = lane & 15, g = lane >> 4;
    const int T = item * TG + j;     // global tile index
    if (EPI == EPI_RESID) {
        publish_h_tile(P, X, A.next_gain, T, t, g, hcur + v, t < P.M);
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
                    const __amdgpu_buffer_rsrc_t rq = co_rsrc(X.q, 2 * (P.q_plane * 2));
                    const int off = (int)(((size_t)t * P.hd + head * P.dh + p0) * 2);
                    co_st64(rq, off, hi);
                    co_st64(rq, off + (int)(P.q_plane * 2), lo);
                } else if (pos >= 0 && pos < P.seq_pad) {
                    u32x2 kk;
                    kk[0] = pack_bf16x2(out[0], out[1]);
                    kk[1] = pack_bf16x2(out[2], out[3]);
                    const __amdgpu_buffer_rsrc_t rk = co_rsrc(P.kv + kv_k_off(geo, A.layer, b, head), head_bytes);
                    co_st64(rk, (int)(((size_t)pos * P.dh + p0) * 2), kk);
                }
            }
        } else if (t < P.M && pos >= 0 && pos < P.seq_pad) {
            const __amdgpu_buffer_rsrc_t rv = co_rsrc(P.kv + kv_v_off(geo, A.layer, b, head), head_bytes);
#pragma unroll
            for (int r = 0; r < 4; r++)
                co_st16(rv, (int)(kv_v_idx(geo, 16 * ti + 4 * g + r, pos) * 2), f32_to_bf16(v[r]));
        }
    }
}

// Copy the two planes of a row-major activation buffer [M][ld] into LDS in fragment order:
// 16-byte unit ((ks*2 + plane)*4 + g)*M + row holds k = 32 ks + 8 g .. +7 of that row.
#define COPY_ROWS 6
#define COPY_ROWS 6
__device__ __forceinline__ void copy_to_lds(CParams &P, const bf16_t *__restrict__ src, size_t plane, int ld,
                                            char *smem) {
    const int tid = threadIdx.x, M = P.M, ld8 = ld / 8;
    u32x4 *act = reinterpret_cast<u32x4 *>(smem);
    for (int kc = tid; kc < ld8; kc += FUSED_THREADS) {
        const int ks = kc >> 2, g = kc & 3;
        // COPY_ROWS rows x 2 planes in flight per thread: the usual block (k+1 <= 6 rows) takes one memory round trip
        for (int r0 = 0; r0 < M; r0 += COPY_ROWS) {
            u32x4 a[COPY_ROWS][2];
#pragma unroll
            for (int u = 0; u < COPY_ROWS; u++)
                if (r0 + u < M) {
                    const bf16_t *sp = src + (size_t)(r0 + u) * ld + kc * 8;
                    a[u][0] = *reinterpret_cast<const u32x4 *>(sp);
                    a[u][1] = *reinterpret_cast<const u32x4 *>(sp + plane);
                }
#pragma unroll
            for (int u = 0; u < COPY_ROWS; u++)
                if (r0 + u < M) {
                    act[((ks * 2 + 0) * 4 + g) * M + r0 + u] = a[u][0];
                    act[((ks * 2 + 1) * 4 + g) * M + r0 + u] = a[u][1];
                }
        }
    }
}

#define W_RING 32   /* 16-byte fragments per lane held by the weight ring: 32 KB per wave, 256 KB per CU */

// Wave 0 of a workgroup is its service wave: it signals and polls the device-wide barrier, computes
// the row scales, and applies the reduction + epilogue of each work item while the other seven waves
// already stream the next item.  Loads return in order, so a wave with a weight burst in flight would
// see its barrier polls delayed by the whole burst; the service wave never streams weights.
#define STREAM_WAVES (FUSED_WAVES - 1)

// The weight stream of one streaming wave.  It owns the K slice [ks0, ks1) of every work item its
// workgroup takes (item = wg, wg + nwg, ...).  The slice is cut into batches of U k-steps x TG tiles;
// batch n of the wave is batch n % nbpi of its item n / nbpi.  NW batches live in a register ring; the
// loads of batch n + NW are issued right after batch n has been multiplied, so the stream runs ahead
// across item boundaries, and the first NW batches of a phase are issued before the device-wide
// barrier that precedes it (they depend on nothing but the weights).
template <int TG, int U, int NW>
struct WStream {
    const u32x4 *Wp;
    int KS, n_items, wg, nwg, ks0, ks1, nbpi, lane;
    __device__ __forceinline__ void init(const u32x4 *Wp_, int KS_, int n_items_, int wg_, int nwg_) {
        Wp = Wp_;
        KS = KS_;
        n_items = n_items_;
        wg = wg_;
        nwg = nwg_;
        lane = threadIdx.x & 63;
        const int sw = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) - 1;   // streaming wave index (scalar); -1 for the service wave
        ks0 = sw < 0 ? 0 : KS * sw / STREAM_WAVES;
        ks1 = sw < 0 ? 0 : KS * (sw + 1) / STREAM_WAVES;
        const int nb_max = ((KS + STREAM_WAVES - 1) / STREAM_WAVES + U - 1) / U;   // same for every wave
        nbpi = (nb_max + NW - 1) / NW * NW;      // padded: the ring turns a whole number of times per item
        if (nbpi == 0) nbpi = NW;
    }
    // load cursor: the next batch to issue is batch l_b of item l_item
    int l_item, l_b;
    __device__ __forceinline__ void rewind() {
        l_item = wg;
        l_b = 0;
    }
    // after the first NW batches have been issued (by prefetch(), possibly before the barrier)
    __device__ __forceinline__ void skip_prefetched() {
        l_item = NW == nbpi ? wg + nwg : wg;
        l_b = NW == nbpi ? 0 : NW;
    }
    // issue the loads of the cursor's batch into ring slot `slot` (a constant once the caller's loop is
    // unrolled) and advance the cursor
    __device__ __forceinline__ void load_next(u32x4 (&W)[W_RING], int slot, bool issue = true) {
        const int item = l_item, ks = ks0 + l_b * U;
        if (++l_b == nbpi) {
            l_b = 0;
            l_item += nwg;
        }
        if (item >= n_items || !issue) return;   // stream exhausted (uniform)
        const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < U; u++)
#pragma unroll
            for (int j = 0; j < TG; j++)
                W[(slot * U + u) * TG + j] =
                    (ks + u < ks1) ? __builtin_nontemporal_load(Wp + ((size_t)(item * TG + j) * KS + ks + u) * 64 + lane) : zero;
    }
    // issue ring slots [from, to) of the first NW batches
    __device__ __forceinline__ void prefetch(u32x4 (&W)[W_RING], int from = 0, int to = NW) {
        rewind();
#pragma unroll
        for (int s = 0; s < NW; s++) load_next(W, s, s >= from && s < to);
    }
};

// One weight-streaming GEMM phase.
// B_LDS: the activation rows (two bf16 planes) are first copied into LDS in fragment order and the
// whole register ring holds weights.  Otherwise (K too long for LDS) the activations come from L2
// through a two-batch ring that takes the upper half of the registers.
// `prefetched`: the first NW weight batches were already issued into W before the barrier.
template <int TG, int EPI, bool B_LDS, int U, int NW>
__device__ __forceinline__ void gemm_phase(CParams &P, const PhaseBufs &X, const GemmArgs &A, char *smem, int wg, int nwg,
                                           u32x4 (&W)[W_RING], int prefetched) {
    static_assert(NW * U * TG <= (B_LDS ? W_RING : W_RING / 2), "weight ring does not fit");
    static_assert(B_LDS || 4 * U <= W_RING / 2, "activation ring does not fit");
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool service = w == 0;
    const int sw = w - 1;
    const int t = lane & 15, g = lane >> 4;
    const int M = P.M;
    const u32x4 *lds_act = reinterpret_cast<const u32x4 *>(smem);
    f32x4 *red = reinterpret_cast<f32x4 *>(smem + P.lds_red_off);      // [2 buffers][7 waves][TG][64 lanes]
    constexpr int RED_BUF = STREAM_WAVES * 3 * 64;
    if (wg >= A.n_items) return;      // whole workgroup idle in this phase (uniform)
    WStream<TG, U, NW> ws;
    ws.init(A.Wp, A.KS, A.n_items, wg, nwg);
    const bool valid = t < M;
    const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
    const u32x4 *bp = reinterpret_cast<const u32x4 *>(A.bsrc + (size_t)(valid ? t : 0) * A.ldb + 8 * g);
    const size_t bplane16 = A.bplane / 8;
    constexpr int BQ = W_RING / 2;    // activation ring lives in W[BQ ..]: slot*2U + 2u + plane

#define FUSED_LOAD_B(SLOT, BATCH)   /* BATCH >= nbpi: the next item, same K slice */                \
    if (!B_LDS) {                                                                                   \
        const int bq_ = (BATCH) >= ws.nbpi ? (BATCH) - ws.nbpi : (BATCH);                           \
        const int ksb_ = ws.ks0 + bq_ * U;                                                          \
        _Pragma("unroll") for (int u = 0; u < U; u++) {                                             \
            const bool in_ = valid && ksb_ + u < ws.ks1;                                            \
            W[BQ + ((SLOT) * U + u) * 2 + 0] = in_ ? bp[(size_t)(ksb_ + u) * 4] : zero;             \
            W[BQ + ((SLOT) * U + u) * 2 + 1] = in_ ? bp[(size_t)(ksb_ + u) * 4 + bplane16] : zero;  \
        }                                                                                           \
    }
#define FUSED_MMA(SLOT, BSLOT, BATCH)                                                               \
    {                                                                                               \
        const int ksm_ = ws.ks0 + __builtin_amdgcn_readfirstlane(BATCH) * U;                        \
        _Pragma("unroll") for (int u = 0; u < U; u++) {                                             \
            u32x4 bh_ = zero, bl_ = zero;                                                           \
            if (B_LDS) {                                                                            \
                if (valid && ksm_ + u < ws.ks1) {                                                   \
                    bh_ = lds_act[(((ksm_ + u) * 2 + 0) * 4 + g) * M + t];                          \
                    bl_ = lds_act[(((ksm_ + u) * 2 + 1) * 4 + g) * M + t];                          \
                }                                                                                   \
            } else {                                                                                \
                bh_ = W[BQ + ((BSLOT) * U + u) * 2 + 0];                                            \
                bl_ = W[BQ + ((BSLOT) * U + u) * 2 + 1];                                            \
            }                                                                                       \
            _Pragma("unroll") for (int j = 0; j < TG; j++) {                                        \
                const bf16x8 wf_ = __builtin_bit_cast(bf16x8, W[((SLOT) * U + u) * TG + j]);        \
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf_, __builtin_bit_cast(bf16x8, bh_), acc[j], 0, 0, 0); \
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf_, __builtin_bit_cast(bf16x8, bl_), acc[j], 0, 0, 0); \
            }                                                                                       \
        }                                                                                           \
    }

    if (B_LDS) {
        copy_to_lds(P, A.bsrc, A.bplane, A.ldb, smem);
        if (prefetched < NW && !service) ws.prefetch(W, prefetched, NW);
    } else if (!service) {
        FUSED_LOAD_B(0, 0)
        FUSED_LOAD_B(1, 1)
        if (prefetched < NW) ws.prefetch(W, prefetched, NW);
    }
    ws.skip_prefetched();
    // service wave: the first item's residual tiles (they do not change during the phase) and the row scales
    f32x4 hfirst[TG];
#pragma unroll
    for (int j = 0; j < TG; j++) hfirst[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (service) {
        if (EPI == EPI_RESID && valid) {
#pragma unroll
            for (int j = 0; j < TG; j++)
                hfirst[j] = *reinterpret_cast<const f32x4 *>(X.h_in + (size_t)t * P.d + (wg * TG + j) * 16 + 4 * g);
        }
    }
    if (B_LDS) lds_sync();
    // row scale of this lane's row (service wave only; needed at the first epilogue, so it overlaps the
    // streaming): rstd = 1/sqrt(sum of the per-tile sums of squares / d + eps); lane group g adds tiles
    // g, g+4, ... in a fixed order, 16 loads in flight at a time
    float rs_row = 1.0f;
    if (service && A.scaled) {
        // ssq is [row][tile]; lane group g adds tiles [g*per, (g+1)*per) of row t, four at a time, in order
        const int nt = P.d / 16, per = nt / 4;
        const f32x4 *sp = reinterpret_cast<const f32x4 *>(X.ssq_in + (size_t)t * nt + g * per);
        float ss = 0.f;
        for (int c0 = 0; c0 < per / 4; c0 += 16) {
            f32x4 v[16];
#pragma unroll
            for (int u = 0; u < 16; u++) v[u] = (valid && c0 + u < per / 4) ? sp[c0 + u] : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < 16; u++) ss += (v[u][0] + v[u][1]) + (v[u][2] + v[u][3]);
        }
        ss += __shfl_xor(ss, 16, 64);
        ss += __shfl_xor(ss, 32, 64);
        rs_row = rsqrtf(ss / (float)P.d + P.eps);
    }
    ts_mark(P, X, TS_PROLOGUE);
    int parity = 0;
#pragma unroll 1
    for (int item = wg; item < A.n_items; item += nwg, parity ^= 1) {
        f32x4 *rb = red + parity * RED_BUF;
        if (!service) {
            f32x4 acc[TG];
#pragma unroll
            for (int j = 0; j < TG; j++) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
            for (int bb = 0; bb < ws.nbpi; bb += NW) {
#pragma unroll
                for (int sl = 0; sl < NW; sl++) {
                    FUSED_MMA(sl, sl & 1, bb + sl)
                    ws.load_next(W, sl);
                    FUSED_LOAD_B(sl & 1, bb + sl + 2)
                }
            }
#pragma unroll
            for (int j = 0; j < TG; j++) rb[(sw * TG + j) * 64 + lane] = acc[j];
        }
        // partial sums of this item are in red[parity]; the streaming waves go straight on to the next item
        // (which uses the other buffer) while the service wave reduces in a fixed order and applies the epilogue
        lds_sync();
        if (service) {
            if (item + nwg >= A.n_items) ts_mark(P, X, TS_LOOP);
            const float rs = rs_row;
            if (EPI == EPI_SWIGLU) {              // TG == 2: tile 0 = gate, tile 1 = up, same 16 features
                f32x4 gsum = rb[lane], usum = rb[64 + lane];
#pragma unroll
                for (int ww = 1; ww < STREAM_WAVES; ww++) {
                    gsum += rb[(ww * TG) * 64 + lane];
                    usum += rb[(ww * TG + 1) * 64 + lane];
                }
                if (valid) {
                    float f[4];
#pragma unroll
                    for (int r = 0; r < 4; r++) {
                        const float gg = gsum[r] * rs;
                        f[r] = gg / (1.0f + expf(-gg)) * (usum[r] * rs);
                    }
                    u32x2 hi, lo;
                    split4(f, hi, lo);
                    const __amdgpu_buffer_rsrc_t rf = co_rsrc(X.ffn_a, 2 * (P.ffn_plane * 2));
                    const int off = (int)(((size_t)t * P.F + item * 16 + 4 * g) * 2);
                    co_st64(rf, off, hi);
                    co_st64(rf, off + (int)(P.ffn_plane * 2), lo);
                }
            } else {
#pragma unroll
                for (int j = 0; j < TG; j++) {
                    f32x4 sum = rb[j * 64 + lane];
#pragma unroll
                    for (int ww = 1; ww < STREAM_WAVES; ww++) sum += rb[(ww * TG + j) * 64 + lane];
                    sum *= rs;
                    f32x4 hcur = hfirst[j];
                    if (EPI == EPI_RESID && item != wg && valid)
                        hcur = *reinterpret_cast<const f32x4 *>(X.h_in + (size_t)t * P.d + (item * TG + j) * 16 + 4 * g);
                    gemm_epilogue<TG, EPI>(P, X, A, item, j, sum, lane, hcur);
                }
            }
        }
    }
#undef FUSED_LOAD_B
#undef FUSED_MMA
}

#define ATTN_BATCH 16   /* items a workgroup works off before it counts them in */

// Second stage of the attention phase for the n items whose partial states this workgroup has written:
// wait once for all those stores, count every item into its (sequence, head) counter (one lane each),
// and for each head where this workgroup was the last key group to finish, merge all its groups and
// write the attention output.  Doing this once per batch of items, not once per item, keeps the chain
// store acknowledgement -> counter -> partial loads off the per-item path.
template <int DH>
__device__ __forceinline__ void attn_finish(CParams &P, __amdgpu_buffer_rsrc_t ro, const int *s_item, int *s_last, int n) {
    constexpr int PS = DH + 4;
    const int tid = threadIdx.x;
    const size_t part_elems = (size_t)16 * PS;
    stores_acked_sync();    // the partial states of all n items
    if (tid < n) {
        const int item = s_item[tid];
        const int hh = (item / P.kg_max) % P.H, b = item / (P.kg_max * P.H);
        const int nk = max(0, min(P.cache_len[b] + P.m, P.seq_pad));
        const int n_groups = (nk + 255) / 256;
        const unsigned old = __hip_atomic_fetch_add(P.attn_cnt + b * P.H + hh, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last[tid] = (old == (unsigned)(n_groups - 1));
    }
    __syncthreads();
    for (int i = 0; i < n; i++) {
        if (!s_last[i]) continue;           // uniform
        const int item = s_item[i];
        const int hh = (item / P.kg_max) % P.H, b = item / (P.kg_max * P.H);
        const int nk = max(0, min(P.cache_len[b] + P.m, P.seq_pad));
        const int n_groups = (nk + 255) / 256;
        const __amdgpu_buffer_rsrc_t rp =
            co_rsrc(P.attn_part + (size_t)((b * P.H + hh) * P.kg_max) * part_elems, sizeof(float) * part_elems * P.kg_max);
        for (int idx = tid; idx < P.m * (DH / 4); idx += FUSED_THREADS) {
            const int r = idx / (DH / 4), x4 = idx % (DH / 4);
            // eight groups' states in flight together (one memory round trip for the usual case), groups
            // combined in index order
            float mstar = -INFINITY, den = 0.f;
            f32x4 num = f32x4{0.f, 0.f, 0.f, 0.f};
            for (int c0 = 0; c0 < n_groups; c0 += 8) {
                float mc[8], dc[8];
                f32x4 nc[8];
#pragma unroll
                for (int u = 0; u < 8; u++) {
                    const int c = min(c0 + u, n_groups - 1);
                    const int base = (int)(((size_t)c * part_elems + (size_t)r * PS) * 4);
                    mc[u] = co_ld32f(rp, base + DH * 4);
                    dc[u] = co_ld32f(rp, base + (DH + 1) * 4);
                    nc[u] = co_ld128f(rp, base + x4 * 16);
                }
                float mchunk = mstar;
#pragma unroll
                for (int u = 0; u < 8; u++)
                    if (c0 + u < n_groups) mchunk = fmaxf(mchunk, mc[u]);
                const float a = (mstar == -INFINITY) ? 0.f : expf(mstar - mchunk);
                num *= a;
                den *= a;
#pragma unroll
                for (int u = 0; u < 8; u++) {
                    const float wgt = (c0 + u >= n_groups || mc[u] == -INFINITY) ? 0.f : expf(mc[u] - mchunk);
                    num += nc[u] * wgt;
                    den += dc[u] * wgt;
                }
                mstar = mchunk;
            }
            const float inv = den > 0.f ? 1.0f / den : 0.f;
            float o[4] = {num[0] * inv, num[1] * inv, num[2] * inv, num[3] * inv};
            u32x2 hi, lo;
            split4(o, hi, lo);
            const int off = (int)(((size_t)(b * P.m + r) * P.hd + hh * DH + x4 * 4) * 2);
            co_st64(ro, off, hi);
            co_st64(ro, off + (int)(P.q_plane * 2), lo);
        }
        if (tid == 0) __hip_atomic_store(P.attn_cnt + b * P.H + hh, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();        // s_item / s_last may be reused
}

// Block attention for one 16-row tile per sequence (m <= 16).
template <int DH>
__device__ __noinline__ void phase_attn(CParams &P, int layer, char *smem, int wg, int nwg) {
    const PhaseBufs X = make_bufs(P, PH_ATTN, layer, 0);
    constexpr int PS = DH + 4;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int col = lane & 15, g = lane >> 4;
    float *lacc = reinterpret_cast<float *>(smem);              // [8 waves][16 rows][PS]
    // items whose partial state this workgroup has written and not yet counted in (see attn_finish)
    __shared__ int s_item[ATTN_BATCH], s_last[ATTN_BATCH];
    int n_mine = 0;
    const KvGeom geo{P.Bmax, P.H, P.dh, P.seq_pad, P.L, P.kperm};
    const __amdgpu_buffer_rsrc_t ro = co_rsrc(X.attn_o, 2 * (P.q_plane * 2));
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
                    const bf16_t *qp = X.q + (size_t)(b * P.m + col) * P.hd + hh * DH + s * 32 + 8 * g;
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
                vf[dt] = *reinterpret_cast<const u32x4 *>(vc + kv_v_idx(geo, dt * 16 + col, kb + 8 * g));
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
        // the LDS merge area is free again; the partial stores stay in flight while the next item is computed
        lds_sync();
        if (tid == 0) s_item[n_mine] = item;
        if (++n_mine == ATTN_BATCH) {
            attn_finish<DH>(P, ro, s_item, s_last, n_mine);
            n_mine = 0;
        }
    }
    if (n_mine > 0) attn_finish<DH>(P, ro, s_item, s_last, n_mine);
}

__device__ __noinline__ void phase_trace(CParams &P, int slot, int wg, int nwg) {
    const size_t n = (size_t)P.M * P.d;
    for (size_t i = (size_t)wg * FUSED_THREADS + threadIdx.x; i < n; i += (size_t)nwg * FUSED_THREADS)
        P.trace[(size_t)slot * n + i] = P.xh[(size_t)16 * P.d * (P.fresh ? 2 * slot : 0) + i];
}

// Per-phase GEMM shapes: TG tiles per item, U k-steps per batch, NW batches in the register ring.
#define QKV3 3, EPI_QKV, true, 2, 5
#define QKV1 1, EPI_QKV, true, 4, 8
#define OPRJ 1, EPI_RESID, true, 4, 8
#define GUPR 2, EPI_SWIGLU, true, 4, 4
#define DOWN 1, EPI_RESID, false, 4, 4
#define LMH2 2, EPI_LOGITS, true, 4, 4
#define LMH1 1, EPI_LOGITS, true, 4, 8
// the same phases with the activations read from L2 (blocks whose rows do not fit LDS): half the ring for weights
#define QKVL 1, EPI_QKV, false, 4, 4
#define OPRL 1, EPI_RESID, false, 4, 4
#define GUPL 2, EPI_SWIGLU, false, 4, 2
#define LM2L 2, EPI_LOGITS, false, 4, 2
#define LM1L 1, EPI_LOGITS, false, 4, 4

__device__ __forceinline__ GemmArgs gemm_args(CParams &P, const PhaseBufs &X, int phase, int layer) {
    GemmArgs A;
    A.layer = layer;
    A.next_gain = nullptr;
    A.scaled = false;
    A.bsrc = X.hg_in;       // h * gain: input of the projections that follow a norm
    A.bplane = P.hg_plane;
    A.ldb = P.d;
    A.Wp = nullptr;
    A.KS = 0;
    A.n_items = 0;
    if (phase == PH_QKV) {
        A.Wp = P.layers[layer].qkv;
        A.KS = P.d / 32;
        A.scaled = true;
        A.n_items = (3 * P.hd / 16) / P.tg_qkv;
    } else if (phase == PH_O) {
        A.Wp = P.layers[layer].o;
        A.KS = P.hd / 32;
        A.n_items = P.d / 16;
        A.bsrc = X.attn_o;
        A.bplane = P.q_plane;
        A.ldb = P.hd;
        A.next_gain = P.layers[layer].ffn_norm;
    } else if (phase == PH_GU) {
        A.Wp = P.layers[layer].gu;
        A.KS = P.d / 32;
        A.scaled = true;
        A.n_items = P.F / 16;
    } else if (phase == PH_DOWN) {
        A.Wp = P.layers[layer].down;
        A.KS = P.F / 32;
        A.n_items = P.d / 16;
        A.bsrc = X.ffn_a;
        A.bplane = P.ffn_plane;
        A.ldb = P.F;
        A.next_gain = layer + 1 < P.L ? P.layers[layer + 1].attn_norm : P.final_norm;
    } else if (phase == PH_LM) {
        A.Wp = P.lm;
        A.KS = P.d / 32;
        A.scaled = true;
        A.n_items = (P.V / 16) / P.tg_lm;
    }
    return A;
}

// issue the first weight batches of a GEMM phase (nothing for the other phases)
template <bool L2B>
__device__ __forceinline__ void prefetch_phase(CParams &P, int phase, int layer, int wg, int nwg, u32x4 (&W)[W_RING]) {
    if (phase != PH_QKV && phase != PH_O && phase != PH_GU && phase != PH_DOWN && phase != PH_LM) return;
    const PhaseBufs X{};      // only the weight side of the arguments is used here
    const GemmArgs A = gemm_args(P, X, phase, layer);
    if (wg >= A.n_items || threadIdx.x < 64) return;     // wave 0 polls the barrier: see gemm_phase
#define FUSED_PF(SHAPE) FUSED_PF_I(SHAPE)
#define FUSED_PF_I(TGv, EPIv, BLv, Uv, NWv)                  \
    {                                                        \
        WStream<TGv, Uv, NWv> ws;                            \
        ws.init(A.Wp, A.KS, A.n_items, wg, nwg);             \
        ws.prefetch(W, 0, P.pf);                             \
    }
    if (L2B) {
        if (phase == PH_QKV) {
            FUSED_PF(QKVL)
        } else if (phase == PH_O) {
            FUSED_PF(OPRL)
        } else if (phase == PH_GU) {
            FUSED_PF(GUPL)
        } else if (phase == PH_DOWN) {
            FUSED_PF(DOWN)
        } else {
            if (P.tg_lm == 2) FUSED_PF(LM2L) else FUSED_PF(LM1L)
        }
    } else if (phase == PH_QKV) {
        if (P.tg_qkv == 3) FUSED_PF(QKV3) else FUSED_PF(QKV1)
    } else if (phase == PH_O) {
        FUSED_PF(OPRJ)
    } else if (phase == PH_GU) {
        FUSED_PF(GUPR)
    } else if (phase == PH_DOWN) {
        FUSED_PF(DOWN)
    } else {
        if (P.tg_lm == 2) FUSED_PF(LMH2) else FUSED_PF(LMH1)
    }
#undef FUSED_PF
#undef FUSED_PF_I
}

template <int DH, bool L2B>
__device__ __forceinline__ void run_phase(CParams &P, const PhaseBufs &X, int phase, int layer, char *smem, int wg, int nwg, u32x4 (&W)[W_RING],
                          int prefetched) {
    if (phase == PH_EMBED) {
        phase_embed(P, wg, nwg);
    } else if (phase == PH_ATTN) {
        phase_attn<DH>(P, layer, smem, wg, nwg);
    } else if (phase == PH_TRACE) {
        phase_trace(P, layer, wg, nwg);
    } else {
        const GemmArgs A = gemm_args(P, X, phase, layer);
        if (L2B) {
            if (phase == PH_QKV) {
                gemm_phase<QKVL>(P, X, A, smem, wg, nwg, W, prefetched);
            } else if (phase == PH_O) {
                gemm_phase<OPRL>(P, X, A, smem, wg, nwg, W, prefetched);
            } else if (phase == PH_GU) {
                gemm_phase<GUPL>(P, X, A, smem, wg, nwg, W, prefetched);
            } else if (phase == PH_DOWN) {
                gemm_phase<DOWN>(P, X, A, smem, wg, nwg, W, prefetched);
            } else if (phase == PH_LM) {
                if (P.tg_lm == 2)
                    gemm_phase<LM2L>(P, X, A, smem, wg, nwg, W, prefetched);
                else
                    gemm_phase<LM1L>(P, X, A, smem, wg, nwg, W, prefetched);
            }
        } else if (phase == PH_QKV) {
            if (P.tg_qkv == 3)
                gemm_phase<QKV3>(P, X, A, smem, wg, nwg, W, prefetched);
            else
                gemm_phase<QKV1>(P, X, A, smem, wg, nwg, W, prefetched);
        } else if (phase == PH_O) {
            gemm_phase<OPRJ>(P, X, A, smem, wg, nwg, W, prefetched);
        } else if (phase == PH_GU) {
            gemm_phase<GUPR>(P, X, A, smem, wg, nwg, W, prefetched);
        } else if (phase == PH_DOWN) {
            gemm_phase<DOWN>(P, X, A, smem, wg, nwg, W, prefetched);
        } else if (phase == PH_LM) {
            if (P.tg_lm == 2)
                gemm_phase<LMH2>(P, X, A, smem, wg, nwg, W, prefetched);
            else
                gemm_phase<LMH1>(P, X, A, smem, wg, nwg, W, prefetched);
        }
    }
}

// one launch per phase
template <int DH, bool L2B>
__global__ __launch_bounds__(FUSED_THREADS, 1) void k_fused_phase(const FusedParams P_arg, int phase, int layer) {
    extern __shared__ __align__(16) char smem[];
    CParams &P = P_arg;
    u32x4 W[W_RING];
    const PhaseBufs X = make_bufs(P, phase, layer, 0);
    run_phase<DH, L2B>(P, X, phase, layer, smem, blockIdx.x, gridDim.x, W, 0);
}

// the whole forward in one launch
template <int DH, bool L2B>
__global__ __launch_bounds__(FUSED_THREADS, 1) void k_verify_persistent(const FusedParams P_arg) {
    extern __shared__ __align__(16) char smem[];
    CParams &P = P_arg;
    const int wg = blockIdx.x, nwg = gridDim.x;
    unsigned epoch = P.bar_base;             // device-wide barriers completed before this launch
    u32x4 W[W_RING];                             // weight ring, carried across phases
    int ts_slot = 0;
    // Lines an earlier launch left in this XCD's L2 or this CU's L1 may be stale now (other XCDs have
    // rewritten the exchange buffers and cache rows since): drop them once, before the first barrier.
    if (threadIdx.x == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    // run a phase, start streaming the next phase's weights, then wait for everyone
#define FUSED_STEP(PHASE, LAYER, PRE, NEXT_PHASE, NEXT_LAYER)          \
    FUSED_STEP_I(PHASE, LAYER, PRE, NEXT_PHASE, NEXT_LAYER, ((PHASE) != PH_EMBED && (PHASE) != PH_ATTN))
#define FUSED_STEP_I(PHASE, LAYER, PRE, NEXT_PHASE, NEXT_LAYER, GEMM)  \
    {                                                                  \
        const PhaseBufs X = make_bufs(P, PHASE, LAYER, ts_slot);       \
        ts_mark(P, X, TS_START);                                       \
        run_phase<DH, L2B>(P, X, PHASE, LAYER, smem, wg, nwg, W, (PRE) ? P.pf : 0); \
        ts_mark(P, X, TS_EPILOGUE);                                    \
        grid_arrive(P, ++epoch, GEMM);                                 \
        if (P.arrive_first) lds_sync();   /* the flag store is issued before this compute unit's prefetch burst */ \
        prefetch_phase<L2B>(P, NEXT_PHASE, NEXT_LAYER, wg, nwg, W);         \
        grid_wait(P, epoch);                                           \
        ts_mark(P, X, TS_BARRIER);                                     \
        ts_slot += TS_PER_PHASE;                                       \
    }
    FUSED_STEP(PH_EMBED, 0, false, PH_QKV, 0)
    if (P.trace) phase_trace(P, 0, wg, nwg);
    for (int l = 0; l < P.L; l++) {
        FUSED_STEP(PH_QKV, l, true, PH_ATTN, l)
        // the ring is empty here: say so, or its registers stay reserved through the attention phase
#pragma unroll
        for (int i = 0; i < W_RING; i++) W[i] = u32x4{0u, 0u, 0u, 0u};
        FUSED_STEP(PH_ATTN, l, false, PH_O, l)
        FUSED_STEP(PH_O, l, true, PH_GU, l)
        FUSED_STEP(PH_GU, l, true, PH_DOWN, l)
        if (l + 1 < P.L) {
            FUSED_STEP(PH_DOWN, l, true, PH_QKV, l + 1)
        } else {
            FUSED_STEP(PH_DOWN, l, true, PH_LM, 0)
        }
        if (P.trace) phase_trace(P, l + 1, wg, nwg);
    }
#undef FUSED_STEP
#undef FUSED_STEP_I
    {
        const PhaseBufs X = make_bufs(P, PH_LM, 0, ts_slot);
        ts_mark(P, X, TS_START);
        run_phase<DH, L2B>(P, X, PH_LM, 0, smem, wg, nwg, W, P.pf);
        ts_mark(P, X, TS_EPILOGUE);
    }
}

// ------------------------------------------------------------------------------- host side

struct FusedState {
    FusedLayer *layers = nullptr;
    float *cs = nullptr;
    unsigned *attn_cnt = nullptr;
    unsigned char *bar = nullptr;
    int bar_scalar = 0;
    int arrive_first = 0;   // tuning knob (env CSD_FUSED_ARRIVE_FIRST): holding the burst back cost 1 % with the present barrier
    unsigned *err = nullptr;
    unsigned bar_epoch = 0;
    int grid = 0, kg_max = 0, tg_qkv = 1, tg_lm = 1;
    size_t lds_bytes = 0;
    int lds_red_off = 0, lds_rstd_off = 0;
    float *xh = nullptr, *xssq = nullptr;
    bf16_t *xhg = nullptr, *xq = nullptr, *xattn = nullptr, *xffn = nullptr;
    int m_limit = 0;       // most rows B*m whose activation fragments fit LDS
    int m_limit_l2b = 0;   // most rows of the variant that reads them from L2 instead
    int fresh = 1;     // tuning knob (env CSD_FUSED_FRESH)
    int pf = 64;       // tuning knob (env CSD_FUSED_PF): ring slots prefetched across a barrier
    int mode = 2;      // 0: off, 1: one launch per phase, 2: persistent
};

// Barrier flags live in uncached device memory.  Such memory is never freed once a kernel has read it
// (tensors allocated after such a free have held wrong values on this platform): buffers of destroyed
// models go back to a process-wide pool and are handed out again.
static std::mutex g_flag_pool_mutex;
static std::vector<void *> g_flag_pool;
static int32_t flag_buffer_acquire(void **p, hipStream_t st) {
    {
        std::lock_guard<std::mutex> lock(g_flag_pool_mutex);
        if (!g_flag_pool.empty()) {
            *p = g_flag_pool.back();
            g_flag_pool.pop_back();
        } else {
            *p = nullptr;
        }
    }
    if (!*p) CSD_HIP(hipExtMallocWithFlags(p, BAR_BYTES, hipDeviceMallocUncached));
    CSD_HIP(hipMemsetAsync(*p, 0, BAR_BYTES, st));
    return CSD_OK;
}
static void flag_buffer_release(void *p) {
    std::lock_guard<std::mutex> lock(g_flag_pool_mutex);
    g_flag_pool.push_back(p);
}

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
    // CSD_PATH = persistent | phases | multikernel picks the path; unset: multikernel.  The single-launch
    // kernel pays a device-wide barrier per phase (and an idle memory system during its attention phase)
    // where the multi-kernel path pays a launch per kernel; measured per verify step, 7B shape, 6 rows:
    // 3.80 ms against 3.68 ms; 160M shape (latency-bound either way): 0.78 against 0.55 ms.
    const char *e = getenv("CSD_PATH");
    int mode = 0;
    if (e && strcmp(e, "persistent") == 0) mode = 2;
    if (e && strcmp(e, "phases") == 0) mode = 1;
    if (mode == 0) return CSD_OK;
    int dev = 0, cus = 0, lds_max = 0;
    CSD_HIP(hipGetDevice(&dev));
    CSD_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    CSD_HIP(hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
    const int d = c.d_model, hd = mod->hd, F = c.d_ffn, V = c.vocab, dh = c.head_dim;
    // LDS: activation fragments M * max(d, hd) * 4 bytes (or the attention merge area), reduction scratch
    // (8 waves x 3 tiles x 1 KB), rstd[16]
    const int red_bytes = 2 * (FUSED_WAVES - 1) * 3 * 64 * 16;   // two buffers of 7 waves x 3 tiles x 1 KB
    const int attn_bytes = FUSED_WAVES * 16 * (dh + 4) * 4;
    const int kmax = d > hd ? d : hd;
    int m_limit = 16;
    while (m_limit > 0 && (size_t)m_limit * kmax * 4 + red_bytes + 256 > (size_t)lds_max) m_limit--;
    if (m_limit < 1 || attn_bytes + red_bytes + 256 > lds_max) return CSD_OK;
    if (d % 256 || hd % 32 || F % 32 || V % 16 || (F / 16) < 1) return CSD_OK;
    FusedState *fs = new FusedState();
    fs->mode = mode;
    if (const char *e = getenv("CSD_FUSED_FRESH")) fs->fresh = atoi(e) ? 1 : 0;
    if (const char *e = getenv("CSD_FUSED_ARRIVE_FIRST")) fs->arrive_first = atoi(e) ? 1 : 0;
    if (const char *e = getenv("CSD_FUSED_PF")) fs->pf = atoi(e) < 0 ? 0 : atoi(e);
    if (const char *e = getenv("CSD_FUSED_M_LDS")) m_limit = atoi(e) < m_limit ? (atoi(e) < 1 ? 1 : atoi(e)) : m_limit;   // test knob
    fs->m_limit = m_limit < mod->m_max ? m_limit : mod->m_max;
    // off unless asked for: from 9 rows on the multi-kernel path with its tall-block GEMMs is faster
    fs->m_limit_l2b = getenv("CSD_FUSED_L2B") ? (16 < mod->m_max ? 16 : mod->m_max) : 0;
    const int m_cap = fs->m_limit;
    size_t act_bytes = (size_t)m_cap * kmax * 4;
    if (act_bytes < (size_t)attn_bytes) act_bytes = attn_bytes;
    fs->lds_red_off = (int)((act_bytes + 255) / 256 * 256);
    fs->lds_rstd_off = fs->lds_red_off + red_bytes;
    fs->lds_bytes = (size_t)fs->lds_rstd_off + 256;
    fs->grid = cus < BAR_MAX_WG ? cus : BAR_MAX_WG;
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
    // exchange buffers: one instance per producing phase (see FusedParams), 16 rows each
    const size_t L = (size_t)c.n_layers, slots = 2 * L + 1;
    if ((rc = fused_alloc(mod, (void **)&fs->xh, sizeof(float) * slots * 16 * d, true, st)) != CSD_OK) return rc;
    if ((rc = fused_alloc(mod, (void **)&fs->xhg, sizeof(bf16_t) * slots * 2 * 16 * d, true, st)) != CSD_OK) return rc;
    if ((rc = fused_alloc(mod, (void **)&fs->xssq, sizeof(float) * slots * 16 * (d / 16), true, st)) != CSD_OK) return rc;
    if ((rc = fused_alloc(mod, (void **)&fs->xq, sizeof(bf16_t) * L * 2 * 16 * hd, true, st)) != CSD_OK) return rc;
    if ((rc = fused_alloc(mod, (void **)&fs->xattn, sizeof(bf16_t) * L * 2 * 16 * hd, true, st)) != CSD_OK) return rc;
    if ((rc = fused_alloc(mod, (void **)&fs->xffn, sizeof(bf16_t) * L * 2 * 16 * F, true, st)) != CSD_OK) return rc;
    if ((rc = fused_alloc(mod, (void **)&fs->attn_cnt, sizeof(unsigned) * c.max_batch * c.n_heads, true, st)) != CSD_OK) return rc;
    if (getenv("CSD_FUSED_VECTOR_POLL")) {
        if ((rc = fused_alloc(mod, (void **)&fs->bar, BAR_BYTES, true, st)) != CSD_OK) return rc;
    } else {
        if ((rc = flag_buffer_acquire((void **)&fs->bar, st)) != CSD_OK) return rc;
        fs->bar_scalar = 1;
    }
    // the flags of the workgroups that exist start at the bit of barrier 0, all others stay 0
    for (int r = 0; r < BAR_REPLICAS; r++) CSD_HIP(hipMemsetAsync(fs->bar + (size_t)r * BAR_REPLICA_STRIDE, 0x01, fs->grid, st));
    if ((rc = fused_alloc(mod, (void **)&fs->err, 256, true, st)) != CSD_OK) return rc;
    // attention partials: [Bmax][H][kg_max][16][dh+4]; reuse the model's buffer when large enough
    const size_t need = sizeof(float) * (size_t)c.max_batch * c.n_heads * fs->kg_max * 16 * (dh + 4);
    if ((rc = fused_alloc(mod, (void **)&mod->fused_attn_part, need, false, st)) != CSD_OK) return rc;
    const void *kernels[4];
    if (dh == 128) {
        kernels[0] = (const void *)k_verify_persistent<128, false>;
        kernels[1] = (const void *)k_verify_persistent<128, true>;
        kernels[2] = (const void *)k_fused_phase<128, false>;
        kernels[3] = (const void *)k_fused_phase<128, true>;
    } else {
        kernels[0] = (const void *)k_verify_persistent<64, false>;
        kernels[1] = (const void *)k_verify_persistent<64, true>;
        kernels[2] = (const void *)k_fused_phase<64, false>;
        kernels[3] = (const void *)k_fused_phase<64, true>;
    }
    for (const void *kfn : kernels)
        CSD_HIP(hipFuncSetAttribute(kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)fs->lds_bytes));
    mod->fused = fs;
    return CSD_OK;
}

void csd_fused_free(csd_model *mod) {
    FusedState *fs = (FusedState *)mod->fused;
    if (fs && fs->bar_scalar && fs->bar) flag_buffer_release(fs->bar);
    delete fs;
    mod->fused = nullptr;
}

bool csd_fused_eligible(const csd_model *mod, int32_t B, int32_t m) {
    const FusedState *fs = (const FusedState *)mod->fused;
    // blocks whose rows fit LDS take the main kernel, blocks of up to 16 rows the variant that reads the
    // activations from L2
    return fs && B * m <= (fs->m_limit_l2b > fs->m_limit ? fs->m_limit_l2b : fs->m_limit) && B * m <= 16 && m <= 16;
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
    const bool l2b = P.M > fs->m_limit;        // the rows do not fit LDS
    P.tg_qkv = l2b ? 1 : fs->tg_qkv;
    P.tg_lm = fs->tg_lm;
    P.pf = fs->pf;
    P.fresh = fs->fresh;
    P.lds_red_off = fs->lds_red_off;
    P.lds_rstd_off = fs->lds_rstd_off;
    P.xh = fs->xh;
    P.xhg = fs->xhg;
    P.xssq = fs->xssq;
    P.xq = fs->xq;
    P.xattn = fs->xattn;
    P.xffn = fs->xffn;
    P.hg_plane = (size_t)16 * c.d_model;
    P.q_plane = (size_t)16 * mod->hd;
    P.ffn_plane = (size_t)16 * c.d_ffn;
    P.eps = c.rms_eps;
    P.scale = 1.0f / sqrtf((float)c.head_dim);
    P.theta = c.rope_theta;
    P.tokens = tokens;
    P.cache_len = cache_len;
    P.embed = (const bf16_t *)mod->embed;
    P.layers = fs->layers;
    P.final_norm = mod->final_norm;
    P.lm = (const u32x4 *)mod->lm.data;
    P.cs = fs->cs;
    P.kv = (bf16_t *)kv;
    P.attn_part = mod->fused_attn_part;
    P.attn_cnt = fs->attn_cnt;
    P.logits = logits;
    P.bar = fs->bar;
    P.bar_scalar = fs->bar_scalar;
    P.arrive_first = fs->arrive_first;
    P.err = fs->err;
    P.trace = mod->trace;
    P.ts = (unsigned long long *)mod->fused_ts;
    const dim3 grid(fs->grid), block(FUSED_THREADS);
    if (fs->mode == 2) {
        P.bar_base = fs->bar_epoch;
        fs->bar_epoch += (unsigned)(1 + 5 * c.n_layers);
        ProfScope ps(mod, st, CSD_PROF_GEMM);
        if (c.head_dim == 128 && !l2b)
            hipLaunchKernelGGL((k_verify_persistent<128, false>), grid, block, fs->lds_bytes, st, P);
        else if (c.head_dim == 128)
            hipLaunchKernelGGL((k_verify_persistent<128, true>), grid, block, fs->lds_bytes, st, P);
        else if (!l2b)
            hipLaunchKernelGGL((k_verify_persistent<64, false>), grid, block, fs->lds_bytes, st, P);
        else
            hipLaunchKernelGGL((k_verify_persistent<64, true>), grid, block, fs->lds_bytes, st, P);
        CSD_LAUNCH_CHECK();
        return CSD_OK;
    }
    P.bar_base = 0;
    auto launch = [&](int phase, int layer, int cls) -> int32_t {
        ProfScope ps(mod, st, cls);
        if (c.head_dim == 128 && !l2b)
            hipLaunchKernelGGL((k_fused_phase<128, false>), grid, block, fs->lds_bytes, st, P, phase, layer);
        else if (c.head_dim == 128)
            hipLaunchKernelGGL((k_fused_phase<128, true>), grid, block, fs->lds_bytes, st, P, phase, layer);
        else if (!l2b)
            hipLaunchKernelGGL((k_fused_phase<64, false>), grid, block, fs->lds_bytes, st, P, phase, layer);
        else
            hipLaunchKernelGGL((k_fused_phase<64, true>), grid, block, fs->lds_bytes, st, P, phase, layer);
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
