// Softmax per position and the speculative-sampling review: accept / resample / extra token
// (Section 2), lenience and the greedy rule (Section 3.1).  One workgroup per sequence.
//
// Every fp32 step that decides an integer is a single rounded IEEE operation (__fmul_rn,
// __fsub_rn: never fused), and the draw is exact integer arithmetic on 40-bit fixed-point
// weights summed in increasing token id, so the outputs do not depend on reduction order.
#include "csd_internal.h"

#pragma clang fp contract(off)

#define ACC_THREADS 1024

// floor(r * 2^40) for a finite fp32 r in [0, 2^24): exact, by shifting the significand
__device__ __forceinline__ unsigned long long fixed40(float r) {
    const uint32_t bits = __float_as_uint(r);
    if ((int32_t)bits <= 0) return 0ull;                    // zero or negative
    const int e = (int)(bits >> 23);                        // sign is 0 here
    if (e == 0) return 0ull;                                // subnormal: below 2^-126
    const unsigned long long mant = (unsigned long long)((bits & 0x7FFFFFu) | 0x800000u);
    const int shift = e - 150 + 40;                         // value = mant * 2^(e-150)
    if (shift >= 0) return shift > 39 ? 0xFFFFFFFFFFFFFFFFull : (mant << shift);
    return shift <= -24 ? 0ull : (mant >> (-shift));
}

// The same number for r in [0, 2^12), without branches or 64-bit shifts, as h * 2^20 + l: h = floor(r * 2^20) (a
// power-of-two scaling and a truncation, both exact), what is left of r * 2^20 is below one and exact as well
// (a float minus its own integer part), and its first 20 binary places are l.  Negative values and NaN give 0.
__device__ __forceinline__ void fixed40_parts(float r, uint32_t &h, uint32_t &l) {
    const float a = fmaxf(r, 0.0f) * 0x1p20f;
    h = (uint32_t)a;
    l = (uint32_t)((a - (float)h) * 0x1p20f);
}
__device__ __forceinline__ unsigned long long fixed40_small(float r) {
    uint32_t h, l;
    fixed40_parts(r, h, l);
    return (unsigned long long)h * (1u << 20) + l;
}

// residual weight of token v at a rejected position: max(0, l*p_v - q_v) in fp32, or p_v itself
__device__ __forceinline__ float weight_at(const float *__restrict__ prow, const float *__restrict__ qrow, int x,
                                           float lenience, bool residual, int v) {
    const float pv = prow[v];
    if (!residual) return pv;
    const float lp = __fmul_rn(lenience, pv);
    const float qv = qrow ? qrow[v] : (v == x ? 1.0f : 0.0f);
    const float df = __fsub_rn(lp, qv);
    return df > 0.0f ? df : 0.0f;
}

struct ArgMax {
    float v;
    int i;
};
__device__ __forceinline__ ArgMax better(ArgMax a, ArgMax b) {     // larger value; ties: smaller index
    return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a;
}

__device__ int block_argmax(const float *__restrict__ row, int V, ArgMax *red) {
    ArgMax best = {-INFINITY, 0x7FFFFFFF};
    for (int v = threadIdx.x; v < V; v += blockDim.x) {
        const float x = row[v];
        // NaN never wins; the first finite-or-inf value does
        if (x > best.v || (x == best.v && v < best.i)) best = {x, v};
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        ArgMax other = {__shfl_xor(best.v, o, 64), __shfl_xor(best.i, o, 64)};
        best = better(best, other);
    }
    const int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = best;
    __syncthreads();
    ArgMax t = red[0];
    for (int i = 1; i < nw; i++) t = better(t, red[i]);
    return t.i == 0x7FFFFFFF ? 0 : t.i;
}

// Sum of the fixed-point weights of tokens [v0, v1) (v0 a multiple of 4): 16-byte loads when the rows
// allow it.  Exact integer arithmetic, so the grouping does not matter.
__device__ __forceinline__ unsigned long long range_weight(const float *__restrict__ prow, const float *__restrict__ qrow,
                                                           int x, float lenience, bool residual, int v0, int v1, bool vec) {
    unsigned long long sum = 0ull;
    int v = v0;
    if (vec) {
        for (; v + 4 <= v1; v += 4) {
            const float4 pv = *reinterpret_cast<const float4 *>(prow + v);
            float w[4] = {pv.x, pv.y, pv.z, pv.w};
            if (residual) {
                float qv[4] = {0.f, 0.f, 0.f, 0.f};
                if (qrow) {
                    const float4 t = *reinterpret_cast<const float4 *>(qrow + v);
                    qv[0] = t.x, qv[1] = t.y, qv[2] = t.z, qv[3] = t.w;
                } else if (x >= v && x < v + 4) {
                    qv[x - v] = 1.0f;
                }
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const float df = __fsub_rn(__fmul_rn(lenience, w[i]), qv[i]);
                    w[i] = df > 0.0f ? df : 0.0f;
                }
            }
#pragma unroll
            for (int i = 0; i < 4; i++) sum += fixed40(w[i]);
        }
    }
    for (; v < v1; v++) sum += fixed40(weight_at(prow, qrow, x, lenience, residual, v));
    return sum;
}

// Exclusive prefix of one 64-bit value per thread over the block, in thread order, and the block total.
__device__ __forceinline__ unsigned long long block_exclusive_scan(unsigned long long mine, unsigned long long *wave_tot,
                                                                   unsigned long long &total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    unsigned long long incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned long long up = __shfl_up(incl, o, 64);
        if (lane >= o) incl += up;
    }
    __syncthreads();
    if (lane == 63) wave_tot[w] = incl;
    __syncthreads();
    unsigned long long before = 0ull;
    total = 0ull;
    for (int i = 0; i < nw; i++) {
        if (i == w) before = total;
        total += wave_tot[i];
    }
    return before + incl - mine;
}

// The review of one sequence by one workgroup (every thread calls it; the result is valid in every thread).
// pb: reviewer rows [k+1][V]; qb: draft rows [k][V] or null; q_onehot: [k] flags or null; db: drafts [k];
// ua: [k] uniforms of the acceptance tests; us: the uniform of the draw.
struct AcceptShared {
    ArgMax red_am[ACC_THREADS / 64];
    unsigned long long wave_tot[ACC_THREADS / 64];
    int s_n, s_tok;
};
__device__ __forceinline__ void accept_core(AcceptShared &S, const float *__restrict__ pb, const float *__restrict__ qb,
                                            const uint8_t *__restrict__ q_onehot, const int32_t *__restrict__ db,
                                            const float *__restrict__ ua, float us, int32_t k, int32_t V, float lenience,
                                            int32_t mode, int &n_out, int &tok_out) {
    if (mode == CSD_MODE_GREEDY) {
        int n = 0, am = 0;
        for (; n <= k; n++) {
            am = block_argmax(pb + (size_t)n * V, V, S.red_am);
            if (n == k) break;
            const int x = db[n];
            bool ok = (x == am);
            if (!ok && lenience > 1.0f && x >= 0 && x < V) {
                const bool dense = qb && !(q_onehot && q_onehot[n]);
                const float qx = dense ? qb[(size_t)n * V + x] : 1.0f;
                ok = qx <= __fmul_rn(lenience, pb[(size_t)n * V + x]);
            }
            if (!ok) break;
        }
        n_out = n;
        tok_out = am;
        return;
    }
    // acceptance tests of all k positions at once (one lane each); the first failure ends the prefix
    if (threadIdx.x < 64) {
        int n = k;
        for (int base = 0; base < k && n == k; base += 64) {
            const int i = base + (int)threadIdx.x;
            bool ok = true;
            if (i < k) {
                const int x = db[i];
                ok = false;
                if (x >= 0 && x < V) {                           // an invalid draft id is a rejection
                    const bool dense = qb && !(q_onehot && q_onehot[i]);
                    const float qx = dense ? qb[(size_t)i * V + x] : 1.0f;
                    const float lhs = __fmul_rn(ua[i], qx);
                    const float rhs = __fmul_rn(lenience, pb[(size_t)i * V + x]);
                    ok = lhs < rhs;
                }
            }
            const unsigned long long bad = __ballot(!ok);
            if (bad) n = base + __ffsll((long long)bad) - 1;
        }
        if (threadIdx.x == 0) {
            S.s_n = n;
            S.s_tok = -1;
        }
    }
    __syncthreads();
    const int n = S.s_n;
    const float *prow = pb + (size_t)n * V;
    bool residual = n < k;
    int x = residual ? db[n] : -1;
    const float *qrow = nullptr;
    // a draft id outside [0, V) is a rejection whose replacement is drawn from the reviewer's row itself
    if (residual && (x < 0 || x >= V)) residual = false;
    if (residual && qb && !(q_onehot && q_onehot[n])) qrow = qb + (size_t)n * V;
    const bool vec = ((uintptr_t)prow % 16 == 0) && (!qrow || (uintptr_t)qrow % 16 == 0);

    // thread t owns tokens [v0, v1), a whole number of 4-token groups
    const int chunk = ((V + ACC_THREADS - 1) / ACC_THREADS + 3) / 4 * 4;
    const int v0 = min(V, (int)threadIdx.x * chunk), v1 = min(V, v0 + chunk);
    unsigned long long Z = 0ull, excl = 0ull, mine = 0ull;
    for (int pass = 0; pass < 2; pass++) {
        mine = range_weight(prow, qrow, x, lenience, residual, v0, v1, vec);
        excl = block_exclusive_scan(mine, S.wave_tot, Z);
        if (Z != 0ull || !residual) break;
        residual = false;                                    // all-zero residual: draw from the reviewer's row
    }
    if (Z != 0ull) {                                         // else not a distribution: the token stays -1
        // T = floor(floor(u * 2^24) * Z / 2^24), 128-bit product
        const unsigned long long u24 = fixed40(us) >> 16;
        const unsigned long long hi = __umul64hi(u24, Z), lo = u24 * Z;
        const unsigned long long T = (hi << 40) | (lo >> 24);
        if (T >= excl && T < excl + mine) {                  // exactly one thread owns T
            unsigned long long cum = excl;
            int tok = v1 - 1;
            for (int v = v0; v < v1; v++) {
                cum += fixed40(weight_at(prow, qrow, x, lenience, residual, v));
                if (cum > T) { tok = v; break; }
            }
            S.s_tok = tok;
        }
    }
    __syncthreads();
    n_out = n;
    tok_out = S.s_tok;
}

__global__ __launch_bounds__(ACC_THREADS) void k_accept(
    const float *__restrict__ p, const float *__restrict__ q, const uint8_t *__restrict__ q_onehot,
    const int32_t *__restrict__ draft, int32_t draft_stride, const float *__restrict__ u_acc,
    const float *__restrict__ u_samp, int32_t k, int32_t V, float lenience, int32_t mode,
    int32_t *__restrict__ n_accepted, int32_t *__restrict__ next_token) {
    __shared__ AcceptShared S;
    const int b = blockIdx.x;
    int n, tok;
    accept_core(S, p + (size_t)b * (k + 1) * V, q ? q + (size_t)b * k * V : nullptr, q_onehot, draft + (size_t)b * draft_stride,
                u_acc ? u_acc + (size_t)b * k : nullptr, mode == CSD_MODE_SAMPLE ? u_samp[b] : 0.f, k, V, lenience, mode, n, tok);
    if (threadIdx.x == 0) {
        n_accepted[b] = n;
        next_token[b] = tok;
    }
}

// ------------------------------------------------------------------------------------------------ softmax
//
// p = e_v / sum_v e_v with e_v = exp(x_v / T - max).  The sum is taken exactly: every e_v (in [0, 1]) goes to 40-bit
// fixed point and the integers are added, so the sum, and with it every probability, does not depend on how the
// row is spread over threads.  Two kernels with different layouts (k_softmax, k_review_rows) therefore produce
// the same bits.
#define SM_THREADS 1024
#define SM_PER 32

__device__ __forceinline__ unsigned long long block_sum_u64(unsigned long long v, unsigned long long *red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    const int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    unsigned long long t = 0ull;
    for (int i = 0; i < nw; i++) t += red[i];
    return t;
}
__device__ __forceinline__ float scaled_logit(float x, float inv_t) { return x * inv_t; }
__device__ __forceinline__ float exp_term(float xs, float mx) { return expf(xs - mx); }
// 1 / sum from the fixed-point total (at most 2^15 terms of at most 2^40 each)
__device__ __forceinline__ float recip_of_total(unsigned long long total) {
    return 1.0f / (__ull2float_rn(total) * 0x1p-40f);
}

// one workgroup per row.  Each thread keeps its SM_PER elements in registers between the three steps (rows
// longer than SM_THREADS * SM_PER take the generic loop).
__global__ __launch_bounds__(SM_THREADS) void k_softmax(const float *logits, float *probs, int32_t V, float inv_t) {
    __shared__ float red[SM_THREADS / 64];
    __shared__ unsigned long long red64[SM_THREADS / 64];
    const float *x = logits + (size_t)blockIdx.x * V;
    float *y = probs + (size_t)blockIdx.x * V;
    if (V <= SM_THREADS * SM_PER) {
        float val[SM_PER];
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < SM_PER; i++) {
            const int v = i * SM_THREADS + (int)threadIdx.x;
            val[i] = v < V ? scaled_logit(x[v], inv_t) : -INFINITY;
            mx = fmaxf(mx, val[i]);
        }
        mx = block_max(mx, red);
        uint32_t sh = 0, sl = 0;                    // at most 32 terms of at most 2^20 each
#pragma unroll
        for (int i = 0; i < SM_PER; i++) {
            val[i] = exp_term(val[i], mx);          // exp(-inf) = 0 for the padding
            uint32_t h, l;
            fixed40_parts(val[i], h, l);
            sh += h, sl += l;
        }
        const float r = recip_of_total(block_sum_u64((unsigned long long)sh * (1u << 20) + sl, red64));
#pragma unroll
        for (int i = 0; i < SM_PER; i++) {
            const int v = i * SM_THREADS + (int)threadIdx.x;
            if (v < V) y[v] = val[i] * r;
        }
        return;
    }
    float mx = -INFINITY;
    for (int v = threadIdx.x; v < V; v += blockDim.x) mx = fmaxf(mx, scaled_logit(x[v], inv_t));
    mx = block_max(mx, red);
    unsigned long long s = 0ull;
    for (int v = threadIdx.x; v < V; v += blockDim.x) {
        const float e = exp_term(scaled_logit(x[v], inv_t), mx);
        y[v] = e;
        s += fixed40_small(e);
    }
    const float r = recip_of_total(block_sum_u64(s, red64));
    for (int v = threadIdx.x; v < V; v += blockDim.x) y[v] *= r;
}

int32_t csd_softmax_enqueue(const float *logits, float *probs, int64_t rows, int32_t V, float temperature,
                            hipStream_t st) {
    if (rows <= 0) return CSD_OK;
    hipLaunchKernelGGL(k_softmax, dim3((unsigned)rows), dim3(SM_THREADS), 0, st, logits, probs, V, 1.0f / temperature);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

// ------------------------------------------------------------------------- the review, every row at once
//
// The rule of Section 2 / 3.1 walks the drafts in order, but what a row contributes does not depend on the rows
// before it: whether its draft passes, and which token replaces it if it does not.  So a workgroup per
// (row, sequence) normalises its row in registers (the same arithmetic as k_softmax), tests its own draft, and, if
// the draft fails (or the row is the extra one after the drafts), draws the replacement.  It leaves (passed, token)
// in a record; the last workgroup of a sequence to arrive (a counter) picks the first failing row.  No
// probability is written unless the caller asks for it, rows are read once, and nothing waits on anything.
//
// Wave w holds tokens [4096 w, 4096 w + 4096), and in it lane l holds the 4-token groups at 256 j + 4 l, j = 0..15:
// every load is a contiguous kilobyte per wave, and token order is (wave, j, lane, position in the group), which
// is the order the draw's running sum follows.  The result is that of k_softmax + k_accept bit for bit (exact sums
// on both sides).  V <= RR_THREADS * RR_PER; 512 threads, so that a thread may hold its 64 values and more in registers.
// raw: greedy review with lenience 1, which compares token ids of the arg max of the logits themselves.
#define RR_THREADS 512
#define RR_PER 64
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__global__ __launch_bounds__(RR_THREADS) void k_review_rows(
    const float *__restrict__ logits, float *__restrict__ probs, unsigned long long *__restrict__ recs,
    unsigned *__restrict__ counters, float inv_t, const float *__restrict__ q, const uint8_t *__restrict__ q_onehot,
    const int32_t *__restrict__ draft, int32_t draft_stride, const float *__restrict__ u_acc,
    const float *__restrict__ u_samp, int32_t k, int32_t V, float lenience, int32_t mode, int32_t raw,
    int32_t *__restrict__ n_accepted, int32_t *__restrict__ next_token) {
    constexpr int NG = RR_PER / 4;                               // 4-token groups per thread
    __shared__ float red[RR_THREADS / 64];
    __shared__ unsigned long long red64[RR_THREADS / 64];
    __shared__ ArgMax red_am[RR_THREADS / 64];
    __shared__ int s_tok;
    __shared__ unsigned s_old;
    const int row = blockIdx.x, b = blockIdx.y;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const size_t row_off = ((size_t)b * (k + 1) + row) * V;
    const float *xr = logits + row_off;
    const int vbase = wv * (64 * RR_PER) + 4 * lane;             // token of (group j, position c): vbase + 256 j + c
    // what the test of this row's draft needs, requested first: the draft id leads to two more loads
    const bool has_draft = row < k;
    int xd = -1;
    bool valid = false, dense = false;
    float x_logit = 0.f, qx = 1.0f, ua = 0.f, us = 0.f;
    if (has_draft) {
        xd = draft[(size_t)b * draft_stride + row];
        valid = xd >= 0 && xd < V;                              // an invalid draft id is a rejection
        dense = q && !(q_onehot && q_onehot[row]);
        if (mode == CSD_MODE_SAMPLE) ua = u_acc[(size_t)b * k + row];
    }
    if (mode == CSD_MODE_SAMPLE) us = u_samp[b];
    float val[RR_PER];
#pragma unroll
    for (int j = 0; j < NG; j++) {                               // (V is a multiple of 4 and the rows are 16-byte aligned)
        const int v = vbase + 256 * j;
        float4 t = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
        if (v < V) t = *reinterpret_cast<const float4 *>(xr + v);
        val[4 * j] = t.x, val[4 * j + 1] = t.y, val[4 * j + 2] = t.z, val[4 * j + 3] = t.w;
    }
    if (valid) x_logit = xr[xd];                                // behind the row's loads, which do not wait for the id
    if (valid && dense) qx = q[((size_t)b * k + row) * V + xd];
    if (threadIdx.x == 0) s_tok = -1;

    ArgMax best = {-INFINITY, 0x7FFFFFFF};
    if (raw) {          // arg max of the logits (ties: the smaller id; NaN and the -inf padding never win)
#pragma unroll
        for (int i = 0; i < RR_PER; i++)
            if (val[i] > best.v) best = {val[i], vbase + 256 * (i >> 2) + (i & 3)};
    }
    float px = x_logit, mx = -INFINITY, r = 1.0f;
    if (!raw || probs) {
#pragma unroll
        for (int i = 0; i < RR_PER; i++) {
            val[i] = scaled_logit(val[i], inv_t);
            mx = fmaxf(mx, val[i]);
        }
        mx = block_max(mx, red);
        uint32_t sh = 0, sl = 0;                                 // at most 64 terms of at most 2^20 each
#pragma unroll
        for (int i = 0; i < RR_PER; i++) {
            val[i] = exp_term(val[i], mx);
            uint32_t h, l;
            fixed40_parts(val[i], h, l);
            sh += h, sl += l;
        }
        r = recip_of_total(block_sum_u64((unsigned long long)sh * (1u << 20) + sl, red64));
#pragma unroll
        for (int i = 0; i < RR_PER; i++) val[i] = val[i] * r;
        px = exp_term(scaled_logit(x_logit, inv_t), mx) * r;
        if (probs) {
            float *yr = probs + row_off;
#pragma unroll
            for (int j = 0; j < NG; j++) {
                const int v = vbase + 256 * j;
                if (v < V)
                    *reinterpret_cast<float4 *>(yr + v) = make_float4(val[4 * j], val[4 * j + 1], val[4 * j + 2], val[4 * j + 3]);
            }
        }
    }

    bool ok = false;
    int tok = -1;
    if (mode == CSD_MODE_GREEDY) {
        if (!raw) {
#pragma unroll
            for (int i = 0; i < RR_PER; i++)             // (the padding holds 0 at ids above every real one: it loses ties)
                if (val[i] > best.v) best = {val[i], vbase + 256 * (i >> 2) + (i & 3)};
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            ArgMax other = {__shfl_xor(best.v, o, 64), __shfl_xor(best.i, o, 64)};
            best = better(best, other);
        }
        __syncthreads();
        if (lane == 0) red_am[wv] = best;
        __syncthreads();
        ArgMax t = red_am[0];
        for (int i = 1; i < RR_THREADS / 64; i++) t = better(t, red_am[i]);
        tok = t.i == 0x7FFFFFFF ? 0 : min(t.i, V - 1);
        if (has_draft) {
            ok = xd == tok;
            if (!ok && lenience > 1.0f && valid) ok = qx <= __fmul_rn(lenience, px);
        }
    } else {
        if (has_draft && valid) ok = __fmul_rn(ua, qx) < __fmul_rn(lenience, px);
        if (!ok) {
            // the replacement: from norm(max(0, l p - q)) after a failed test of a valid draft, else from p itself
            bool residual = has_draft && valid;
            const float *qrow = residual && dense ? q + ((size_t)b * k + row) * V : nullptr;
            if (residual) {                                  // the weights take the probabilities' place
#pragma unroll
                for (int j = 0; j < NG; j++) {
                    float qv[4] = {0.f, 0.f, 0.f, 0.f};
                    const int v = vbase + 256 * j;
                    if (qrow) {
                        if (v < V) {
                            const float4 t = *reinterpret_cast<const float4 *>(qrow + v);
                            qv[0] = t.x, qv[1] = t.y, qv[2] = t.z, qv[3] = t.w;
                        }
                    } else {
#pragma unroll
                        for (int c = 0; c < 4; c++) qv[c] = v + c == xd ? 1.0f : 0.0f;
                    }
#pragma unroll
                    for (int c = 0; c < 4; c++) {
                        const float df = __fsub_rn(__fmul_rn(lenience, val[4 * j + c]), qv[c]);
                        val[4 * j + c] = df > 0.0f ? df : 0.0f;
                    }
                }
            }
            unsigned long long Z = 0ull, before = 0ull, wave_total = 0ull;
            for (int pass = 0; pass < 2; pass++) {
                unsigned long long mine = 0ull;
#pragma unroll
                for (int i = 0; i < RR_PER; i++) mine += fixed40_small(val[i]);     // weights are at most lenience <= 256
                wave_total = wave_sum_u64(mine);
                __syncthreads();
                if (lane == 0) red64[wv] = wave_total;
                __syncthreads();
                Z = 0ull;
                for (int i = 0; i < RR_THREADS / 64; i++) {
                    if (i == wv) before = Z;
                    Z += red64[i];
                }
                if (Z != 0ull || !residual) break;
                residual = false;                            // all-zero residual: draw from the reviewer's row, rebuilt
#pragma unroll
                for (int j = 0; j < NG; j++) {
                    const int v = vbase + 256 * j;
                    float4 t = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
                    if (v < V) t = *reinterpret_cast<const float4 *>(xr + v);
                    val[4 * j] = exp_term(scaled_logit(t.x, inv_t), mx) * r, val[4 * j + 1] = exp_term(scaled_logit(t.y, inv_t), mx) * r;
                    val[4 * j + 2] = exp_term(scaled_logit(t.z, inv_t), mx) * r, val[4 * j + 3] = exp_term(scaled_logit(t.w, inv_t), mx) * r;
                }
            }
            if (Z != 0ull) {                                 // else not a distribution: the token stays -1
                // T = floor(floor(u * 2^24) * Z / 2^24), 128-bit product
                const unsigned long long u24 = fixed40(us) >> 16;
                const unsigned long long hi = __umul64hi(u24, Z), lo = u24 * Z;
                const unsigned long long T = (hi << 40) | (lo >> 24);
                if (T >= before && T < before + wave_total) {          // exactly one wave owns T
                    unsigned long long run = before;
                    bool found = false;
#pragma unroll
                    for (int j = 0; j < NG; j++) {
                        if (found) continue;                 // (the same in every lane)
                        unsigned long long gj = 0ull;
#pragma unroll
                        for (int c = 0; c < 4; c++) gj += fixed40_small(val[4 * j + c]);
                        const unsigned long long tot = wave_sum_u64(gj);
                        if (T >= run + tot) {
                            run += tot;
                            continue;
                        }
                        found = true;                        // these 256 tokens: the lanes in order
                        unsigned long long incl = gj;
#pragma unroll
                        for (int o = 1; o < 64; o <<= 1) {
                            const unsigned long long up = __shfl_up(incl, o, 64);
                            if (lane >= o) incl += up;
                        }
                        unsigned long long cum = run + incl - gj;
                        if (T >= cum && T < cum + gj) {      // exactly one lane
                            int t = 3;
#pragma unroll
                            for (int c = 2; c >= 0; c--) {   // the first position whose running sum passes T
                                unsigned long long upto = cum;
#pragma unroll
                                for (int cc = 0; cc <= c; cc++) upto += fixed40_small(val[4 * j + cc]);
                                if (upto > T) t = c;
                            }
                            s_tok = min(V - 1, vbase + 256 * j + t);
                        }
                    }
                }
            }
            __syncthreads();
            tok = s_tok;
        }
    }

    // ---- the record of this row, written through to memory and acknowledged before the counter moves
    unsigned long long *rec = recs + (size_t)b * (k + 1);
    if (threadIdx.x == 0) {
        __hip_atomic_store(rec + row, ((unsigned long long)(ok ? 1u : 0u) << 32) | (unsigned)tok, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0)
        s_old = __hip_atomic_fetch_add(counters + b, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (s_old != (unsigned)k || threadIdx.x >= 64) return;
    // ---- last to arrive: the first row whose draft failed decides (device-scope loads: the records come from
    // workgroups on other compute dies)
    int n = k;
    unsigned long long rn = 0ull;
    bool have = false;
    for (int base = 0; base <= k; base += 64) {
        const int i = base + (int)threadIdx.x;
        unsigned long long ri = 1ull << 32;
        if (i <= k) ri = __hip_atomic_load(rec + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long bad = __ballot(i < k && (ri >> 32) == 0ull);
        if (bad) n = base + __ffsll((long long)bad) - 1;
        if (n >= base && n < base + 64) {                    // the deciding row's record is in this batch of lanes
            rn = __shfl(ri, n - base, 64);
            have = true;
        }
        if (bad) break;
    }
    if (threadIdx.x == 0) {
        if (!have) rn = __hip_atomic_load(rec + n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        n_accepted[b] = n;
        next_token[b] = (int32_t)(unsigned)rn;
        __hip_atomic_store(counters + b, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
    }
}

// the kernel takes whole 16-byte groups of four tokens
bool csd_review_rows_fits(const float *logits, const float *probs, const float *q, int32_t V) {
    return V % 4 == 0 && V <= RR_THREADS * RR_PER && (uintptr_t)logits % 16 == 0 && (uintptr_t)probs % 16 == 0 &&
           (uintptr_t)q % 16 == 0;
}

int32_t csd_review_rows_enqueue(const float *logits, float *probs, unsigned long long *recs, unsigned *counters,
                                float temperature, const float *q, const uint8_t *q_onehot, const int32_t *draft,
                                int32_t draft_stride, const float *u_acc, const float *u_samp, int32_t B, int32_t k, int32_t V,
                                float lenience, int32_t mode, int32_t *n_accepted, int32_t *next_token, hipStream_t st) {
    if (B <= 0) return CSD_OK;
    if (!csd_review_rows_fits(logits, probs, q, V)) return CSD_ESHAPE;
    const int32_t raw = mode == CSD_MODE_GREEDY && !(lenience > 1.0f);
    hipLaunchKernelGGL(k_review_rows, dim3(k + 1, B), dim3(RR_THREADS), 0, st, logits, probs, recs, counters,
                       1.0f / (temperature > 0.f ? temperature : 1.0f), q, q_onehot, draft, draft_stride, u_acc, u_samp, k, V,
                       lenience, mode, raw, n_accepted, next_token);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

int32_t csd_accept_enqueue(const float *p, const float *q, const uint8_t *q_onehot, const int32_t *draft,
                           int32_t draft_stride, const float *u_acc, const float *u_samp, int32_t B, int32_t k,
                           int32_t V, float lenience, int32_t mode, int32_t *n_accepted, int32_t *next_token,
                           hipStream_t st) {
    if (B <= 0) return CSD_OK;
    hipLaunchKernelGGL(k_accept, dim3(B), dim3(ACC_THREADS), 0, st, p, q, q_onehot, draft, draft_stride, u_acc, u_samp,
                       k, V, lenience, mode, n_accepted, next_token);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

extern "C" int32_t csd_accept(const float *p, const float *q, const uint8_t *q_onehot, const int32_t *draft,
                              const float *u_acc, const float *u_samp, int32_t B, int32_t k, int32_t V,
                              float lenience, int32_t mode, int32_t *n_accepted, int32_t *next_token, void *stream) {
    if (!p || !n_accepted || !next_token) return CSD_ENULL;
    if (k > 0 && !draft) return CSD_ENULL;
    if (mode == CSD_MODE_SAMPLE && (!u_samp || (k > 0 && !u_acc))) return CSD_ENULL;
    if (B < 0 || k < 0 || V < 1) return CSD_EINVAL;
    if (!(lenience >= 1.0f) || lenience > 256.0f) return CSD_EINVAL;
    if (mode != CSD_MODE_SAMPLE && mode != CSD_MODE_GREEDY) return CSD_EINVAL;
    return csd_accept_enqueue(p, q, q_onehot, draft, k, u_acc, u_samp, B, k, V, lenience, mode, n_accepted,
                              next_token, (hipStream_t)stream);
}

// ------------------------------------------------------------------------------------- review of a tree
//
// Walk down a tree of deterministic candidates (Section 5.1 combines the cascade with tree attention; Appendix B:
// the lead node has eight children): at the current row take the reviewer's own token for the next position (a
// draw from the row with the walk's next uniform, or its arg-max), and if a child of the row carries that token
// keep the child and go on from it; otherwise the token is what the review emits.  One workgroup per sequence; a
// walk step is the draw of a plain review with no drafts.  Rows only have children below them, so the walk ends.
__global__ __launch_bounds__(ACC_THREADS) void k_tree_accept(
    const float *__restrict__ p, const int32_t *__restrict__ tokens, const int32_t *__restrict__ parent,
    const float *__restrict__ u, int32_t m, int32_t V, int32_t mode, int32_t *__restrict__ n_accepted,
    int32_t *__restrict__ path, int32_t *__restrict__ next_token) {
    __shared__ AcceptShared S;
    __shared__ int s_child;
    const int b = blockIdx.x;
    const int32_t *par = parent + (size_t)b * m, *tk = tokens + (size_t)b * m;
    int node = 0, n = 0, tok = -1;
    for (int step = 0; step < m; step++) {
        int unused;
        accept_core(S, p + ((size_t)b * m + node) * V, nullptr, nullptr, nullptr, nullptr,
                    mode == CSD_MODE_SAMPLE ? u[(size_t)b * m + n] : 0.f, 0, V, 1.0f, mode, unused, tok);
        if (threadIdx.x == 0) s_child = 0x7FFFFFFF;
        __syncthreads();
        if (tok >= 0)
            for (int j = node + 1 + (int)threadIdx.x; j < m; j += blockDim.x)
                if (par[j] == node && tk[j] == tok) atomicMin(&s_child, j);    // equal tokens: the lowest row
        __syncthreads();
        const int child = s_child;
        __syncthreads();
        if (child == 0x7FFFFFFF) break;
        if (threadIdx.x == 0) path[(size_t)b * m + n] = child;
        n++;
        node = child;
    }
    if (threadIdx.x == 0) {
        n_accepted[b] = n;
        next_token[b] = tok;
    }
}

extern "C" int32_t csd_tree_accept(const float *p, const int32_t *tokens, const int32_t *parent, const float *u, int32_t B,
                                   int32_t m, int32_t V, int32_t mode, int32_t *n_accepted, int32_t *path, int32_t *next_token,
                                   void *stream) {
    if (!p || !tokens || !parent || !n_accepted || !path || !next_token) return CSD_ENULL;
    if (mode != CSD_MODE_SAMPLE && mode != CSD_MODE_GREEDY) return CSD_EINVAL;
    if (mode == CSD_MODE_SAMPLE && !u) return CSD_ENULL;
    if (B < 0 || m < 1 || V < 1) return CSD_EINVAL;
    if (B == 0) return CSD_OK;
    hipLaunchKernelGGL(k_tree_accept, dim3(B), dim3(ACC_THREADS), 0, (hipStream_t)stream, p, tokens, parent, u, m, V, mode,
                       n_accepted, path, next_token);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

// ------------------------------------------------------------------- device-resident control of the cascade
//
// A review that finds its block in the shared token buffer (Algorithm 1; Sections 3.2, 3.4): the reviewer scores the
// tokens it has not cached yet, ctx[b][cache_len[b] .. ctx_len[b]) = the last kept tokens followed by the drafts in
// flight, keeps a prefix of the drafts, appends its own token, and leaves the sequence, both lengths, the lower
// levels' cache lengths and the draft distributions for the level above updated on the device.  A chain of such
// calls runs a multi-level step with no host synchronisation; what a loop of Algorithm 1 decides on the host
// ("until k_i tokens exist") is a per-sequence condition that the kernels evaluate themselves.

// block[b][i] = ctx[b][cache_len[b] + i] for the rows the reviewer has not cached yet (zero padding up to m_max);
// status[b]: 0 = review, 1 = skipped on request (prefix < 0), 2 = skipped because the state does not fit the call
// (more uncached rows than m_max, a prefix outside the block, draft tables too short)
__global__ void k_gather_block(const int32_t *__restrict__ ctx, int32_t ctx_stride, const int32_t *__restrict__ ctx_len,
                               const int32_t *__restrict__ cache_len, const int32_t *__restrict__ prefix_len, int32_t m_max,
                               const int32_t *__restrict__ q_base, int32_t q_stride, const int32_t *__restrict__ out_base,
                               int32_t out_stride, int32_t *__restrict__ block, int32_t *__restrict__ status) {
    const int b = blockIdx.x;
    const int n = ctx_len[b], cl = cache_len[b], pf = prefix_len[b];
    const int rows = n - cl;
    int st = 0;
    if (pf < 0) st = 1;
    else if (cl < 0 || rows < 1 || rows > m_max || n >= ctx_stride || pf - 1 < cl || pf > n) st = 2;
    else if (q_base && (pf - q_base[b] < 0 || n - q_base[b] > q_stride)) st = 2;
    else if (out_base && (pf - out_base[b] < 0 || n + 1 - out_base[b] > out_stride)) st = 2;
    for (int i = threadIdx.x; i < m_max; i += blockDim.x)
        block[(size_t)b * m_max + i] = (st == 0 && i < rows) ? ctx[(size_t)b * ctx_stride + cl + i] : 0;
    if (threadIdx.x == 0) status[b] = st;
}

struct ReviewArgs {
    int32_t *ctx;
    int32_t ctx_stride;
    int32_t *ctx_len, *cache_len;
    const int32_t *prefix_len;
    const float *q_tab;
    const uint8_t *q_onehot_tab;
    const int32_t *q_base;
    int32_t q_stride;
    const float *u_acc_tab, *u_samp_tab;
    float *out_q_tab;
    uint8_t *out_onehot_tab;
    const int32_t *out_base;
    int32_t out_stride;
    int32_t *lower[4];
    int32_t n_lower;
    int32_t *n_accepted, *next_token;
    const int32_t *status;
    const float *rows;       // reviewer rows [B][m_max][V]: probabilities, or logits for the plain greedy rule
    int32_t m_max, V;
    float lenience;
    int32_t mode;
};

// accept / resample over the drafts in flight, then the commit: the reviewer's own token after the kept drafts, the
// sequence length, this reviewer's cache length, the lower levels' cache lengths (clamped to what is still on the
// path), and the rows the level above will review the emitted tokens against
__global__ __launch_bounds__(ACC_THREADS) void k_review_commit(const ReviewArgs A) {
    __shared__ AcceptShared S;
    const int b = blockIdx.x;
    if (A.status[b] != 0) {
        if (threadIdx.x == 0) {
            if (A.n_accepted) A.n_accepted[b] = -1;
            if (A.next_token) A.next_token[b] = -1;
        }
        return;
    }
    const int n_tok = A.ctx_len[b], cl = A.cache_len[b], pf = A.prefix_len[b];
    const int k = n_tok - pf, row0 = pf - 1 - cl, V = A.V;
    const float *pb = A.rows + ((size_t)b * A.m_max + row0) * V;
    int32_t *seq = A.ctx + (size_t)b * A.ctx_stride;
    const int qi = A.q_base ? pf - A.q_base[b] : 0;
    const float *qb = A.q_tab ? A.q_tab + ((size_t)b * A.q_stride + qi) * V : nullptr;
    const uint8_t *oh = A.q_onehot_tab ? A.q_onehot_tab + (size_t)b * A.q_stride + qi : nullptr;
    const float *ua = A.u_acc_tab ? A.u_acc_tab + (size_t)b * A.ctx_stride + pf : nullptr;
    const float us = (A.mode == CSD_MODE_SAMPLE && A.u_samp_tab) ? A.u_samp_tab[(size_t)b * A.ctx_stride + pf] : 0.f;
    int n, tok;
    accept_core(S, pb, qb, oh, seq + pf, ua, us, k, V, A.lenience, A.mode, n, tok);
    __syncthreads();                                         // every thread has read the lengths it needs
    if (threadIdx.x == 0) {
        seq[pf + n] = tok;
        A.ctx_len[b] = pf + n + 1;
        A.cache_len[b] = pf + n;
        for (int i = 0; i < A.n_lower; i++) A.lower[i][b] = min(A.lower[i][b], pf + n);
        if (A.n_accepted) A.n_accepted[b] = n;
        if (A.next_token) A.next_token[b] = tok;
    }
    // the level above reviews the n + 1 emitted tokens against this reviewer's own rows (sampling); under the greedy
    // rule a draft is its reviewer's arg-max: one-hot
    if (A.out_onehot_tab && threadIdx.x <= n)
        A.out_onehot_tab[(size_t)b * A.out_stride + pf + threadIdx.x - A.out_base[b]] = A.mode == CSD_MODE_SAMPLE ? 0 : 1;
    if (A.out_q_tab && A.mode == CSD_MODE_SAMPLE) {
        float *dst = A.out_q_tab + ((size_t)b * A.out_stride + pf - A.out_base[b]) * V;
        const size_t total = (size_t)(n + 1) * V;
        for (size_t i = threadIdx.x; i < total; i += blockDim.x) dst[i] = pb[i];
    }
}

extern "C" int32_t csd_review_ctx(csd_model *mod, void *kv, const csd_review *r, int32_t B, int32_t m_max, float temperature,
                                  float lenience, int32_t mode, void *stream) {
    if (!r || !r->ctx || !r->ctx_len || !r->cache_len || !r->prefix_len || !r->status) return CSD_ENULL;
    if (!mod || (!kv && !r->ext_rows)) return CSD_ENULL;
    if (B < 1 || m_max < 1 || r->ctx_stride < 2) return CSD_EINVAL;
    if (B > mod->cfg.max_batch || m_max > mod->cfg.max_block) return CSD_ESHAPE;
    if (mode != CSD_MODE_SAMPLE && mode != CSD_MODE_GREEDY) return CSD_EINVAL;
    if (!(lenience >= 1.0f) || lenience > 256.0f) return CSD_EINVAL;
    const bool need_probs = mode == CSD_MODE_SAMPLE || lenience > 1.0f;
    if (need_probs && !r->ext_rows && !(temperature > 0.f)) return CSD_EINVAL;
    if (mode == CSD_MODE_SAMPLE && (!r->u_acc_tab || !r->u_samp_tab)) return CSD_ENULL;
    if ((r->q_tab || r->q_onehot_tab) && (!r->q_base || r->q_stride < 1)) return CSD_EINVAL;
    if ((r->out_q_tab || r->out_onehot_tab) && (!r->out_base || r->out_stride < 1)) return CSD_EINVAL;
    if (r->n_lower < 0 || r->n_lower > 4) return CSD_EINVAL;
    for (int i = 0; i < r->n_lower; i++)
        if (!r->lower_cache_len[i]) return CSD_ENULL;
    hipStream_t st = (hipStream_t)stream;
    const int V = mod->cfg.vocab;
    int32_t *block = mod->review_block;
    hipLaunchKernelGGL(k_gather_block, dim3(B), dim3(64), 0, st, r->ctx, r->ctx_stride, r->ctx_len, r->cache_len, r->prefix_len, m_max,
                       (r->q_tab || r->q_onehot_tab) ? r->q_base : nullptr, r->q_stride,
                       (r->out_q_tab || r->out_onehot_tab) ? r->out_base : nullptr, r->out_stride, block, r->status);
    CSD_LAUNCH_CHECK();
    const float *rows = r->ext_rows;
    if (!rows) {
        int32_t rc;
        float *lg = mod->probs;                               // logits, then probabilities in place
        if ((rc = csd_forward_enqueue(mod, kv, block, r->cache_len, B, m_max, lg, st)) != CSD_OK) return rc;
        if (need_probs && (rc = csd_softmax_enqueue(lg, lg, (int64_t)B * m_max, V, temperature, st)) != CSD_OK) return rc;
        rows = lg;
    }
    ReviewArgs A;
    A.ctx = r->ctx;
    A.ctx_stride = r->ctx_stride;
    A.ctx_len = r->ctx_len;
    A.cache_len = r->cache_len;
    A.prefix_len = r->prefix_len;
    A.q_tab = r->q_tab;
    A.q_onehot_tab = r->q_onehot_tab;
    A.q_base = r->q_base;
    A.q_stride = r->q_stride;
    A.u_acc_tab = r->u_acc_tab;
    A.u_samp_tab = r->u_samp_tab;
    A.out_q_tab = r->out_q_tab;
    A.out_onehot_tab = r->out_onehot_tab;
    A.out_base = r->out_base;
    A.out_stride = r->out_stride;
    for (int i = 0; i < 4; i++) A.lower[i] = i < r->n_lower ? r->lower_cache_len[i] : nullptr;
    A.n_lower = r->n_lower;
    A.n_accepted = r->n_accepted;
    A.next_token = r->next_token;
    A.status = r->status;
    A.rows = rows;
    A.m_max = m_max;
    A.V = V;
    A.lenience = lenience;
    A.mode = mode;
    hipLaunchKernelGGL(k_review_commit, dim3(B), dim3(ACC_THREADS), 0, st, A);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}
