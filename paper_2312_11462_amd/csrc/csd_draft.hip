// Statistical draft model at the bottom of the cascade: Max-Gram matching with a bigram
// fallback (Section 3.3, Appendix A).  Integer-only; one workgroup per sequence.
#include "csd_internal.h"

#define DRAFT_THREADS 256
#define FIT_THREADS 1024

// Max over the block of a 64-bit key; every thread gets the result.
__device__ __forceinline__ unsigned long long block_max_u64(unsigned long long v, unsigned long long *red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        unsigned long long other = __shfl_xor(v, o, 64);
        v = other > v ? other : v;
    }
    const int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    unsigned long long t = red[0];
    for (int i = 1; i < nw; i++) t = red[i] > t ? red[i] : t;
    return t;
}

// Each thread scores candidate match ends e = tid, tid+256, ... <= len-2 by comparing
// backwards against the suffix; the key (match length, ~e) makes the block maximum the
// longest match and, among equals, the left-most end.
__global__ __launch_bounds__(DRAFT_THREADS) void k_bigram_draft(
    const int32_t *__restrict__ ctx, const int32_t *__restrict__ ctx_len, int32_t ctx_stride,
    const int32_t *__restrict__ next_table, int32_t vocab, int32_t k, int32_t max_match,
    int32_t *__restrict__ out_tokens, int32_t *__restrict__ out_match_len) {
    __shared__ unsigned long long red[DRAFT_THREADS / 64];
    const int b = blockIdx.x;
    const int32_t *s = ctx + (size_t)b * ctx_stride;
    int len = ctx_len[b];
    int32_t *out = out_tokens + (size_t)b * k;
    if (len < 1 || len > ctx_stride) {   // device-side guard: no valid context
        for (int j = threadIdx.x; j < k; j += blockDim.x) out[j] = -1;
        if (out_match_len && threadIdx.x == 0) out_match_len[b] = 0;
        return;
    }
    unsigned long long best = 0ull;
    for (int e = threadIdx.x; e <= len - 2; e += blockDim.x) {
        int r = 0;
        while (r <= e && (max_match <= 0 || r < max_match) && s[e - r] == s[len - 1 - r]) r++;
        if (r > 0) {
            unsigned long long key = ((unsigned long long)(uint32_t)r << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)e);
            best = key > best ? key : best;
        }
    }
    best = block_max_u64(best, red);
    const int mlen = (int)(best >> 32);
    if (out_match_len && threadIdx.x == 0) out_match_len[b] = mlen;
    if (mlen == 0) {
        if (threadIdx.x == 0) {          // bigram chain from the last token
            int32_t cur = s[len - 1];
            for (int j = 0; j < k; j++) {
                cur = (cur >= 0 && cur < vocab) ? next_table[cur] : -1;
                out[j] = cur;
            }
        }
        return;
    }
    const int e = (int)(0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull));
    const int period = len - (e + 1);   // >= 1: the sequence extended by its own draft repeats with this period
    for (int j = threadIdx.x; j < k; j += blockDim.x) out[j] = s[e + 1 + (j % period)];
}

// k_bigram_draft that appends its drafts to the context itself (device-resident cascade control): sequences whose
// drafts in flight already number `need` or more (counted from start_len) are left alone.
__global__ __launch_bounds__(DRAFT_THREADS) void k_bigram_draft_append(
    int32_t *__restrict__ ctx, int32_t ctx_stride, int32_t *__restrict__ ctx_len, const int32_t *__restrict__ next_table,
    int32_t vocab, int32_t k, int32_t max_match, const int32_t *__restrict__ gate, uint8_t *__restrict__ q_onehot_tab,
    const int32_t *__restrict__ q_base, int32_t q_stride) {
    __shared__ unsigned long long red[DRAFT_THREADS / 64];
    const int b = blockIdx.x;
    int32_t *s = ctx + (size_t)b * ctx_stride;
    const int len = ctx_len[b];
    bool active = len >= 1 && len + k < ctx_stride && (!gate || gate[b] >= 0);
    if (active && q_onehot_tab && (len - q_base[b] < 0 || len + k - q_base[b] > q_stride)) active = false;
    if (!active) return;                                     // uniform over the workgroup
    unsigned long long best = 0ull;
    for (int e = threadIdx.x; e <= len - 2; e += blockDim.x) {
        int r = 0;
        while (r <= e && (max_match <= 0 || r < max_match) && s[e - r] == s[len - 1 - r]) r++;
        if (r > 0) {
            unsigned long long key = ((unsigned long long)(uint32_t)r << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)e);
            best = key > best ? key : best;
        }
    }
    best = block_max_u64(best, red);                         // (its barriers: every thread has read the context by now)
    const int mlen = (int)(best >> 32);
    int32_t *out = s + len;
    if (mlen == 0) {
        if (threadIdx.x == 0) {                              // bigram chain from the last token
            int32_t cur = s[len - 1];
            for (int j = 0; j < k; j++) {
                cur = (cur >= 0 && cur < vocab) ? next_table[cur] : -1;
                out[j] = cur;
            }
        }
    } else {
        const int e = (int)(0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull));
        const int period = len - (e + 1);                    // sources s[e + 1 ..  len - 1] lie before the drafts
        for (int j = threadIdx.x; j < k; j += blockDim.x) out[j] = s[e + 1 + (j % period)];
    }
    if (q_onehot_tab)
        for (int j = threadIdx.x; j < k; j += blockDim.x) q_onehot_tab[(size_t)b * q_stride + len + j - q_base[b]] = 1;
    if (threadIdx.x == 0) ctx_len[b] = len + k;
}

// gate[b] = ctx_len[b] when sequence b still needs tokens in the loop that started at loop_start[b] (fewer than `need`
// exist) and the enclosing step is itself active (parent_gate null or >= 0); else -1.  A step gated with this value
// reviews drafts that start at that position.
__global__ void k_cascade_gate(const int32_t *__restrict__ ctx_len, const int32_t *__restrict__ loop_start, int32_t need,
                               const int32_t *__restrict__ parent_gate, int32_t B, int32_t *__restrict__ gate) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const bool on = (!parent_gate || parent_gate[b] >= 0) && (!loop_start || ctx_len[b] - loop_start[b] < need);
    gate[b] = on ? ctx_len[b] : -1;
}

// Max-Gram with the haystack apart from the needle (Appendix A's own signature: the encoder's ids are searched
// for the longest suffix of the decoder's ids).  Candidate match ends are all haystack positions; the key is
// the same (match length, ~end).  The continuation is copied while the haystack lasts (out_n_copied of the k
// tokens: what Appendix A returns); the rest chains the bigram table from the last token so far.
__global__ __launch_bounds__(DRAFT_THREADS) void k_maxgram_enc(
    const int32_t *__restrict__ hay, const int32_t *__restrict__ hay_len, int32_t hay_stride,
    const int32_t *__restrict__ needle, const int32_t *__restrict__ needle_len, int32_t needle_stride,
    const int32_t *__restrict__ next_table, int32_t vocab, int32_t k, int32_t max_match,
    int32_t *__restrict__ out_tokens, int32_t *__restrict__ out_match_len, int32_t *__restrict__ out_n_copied) {
    __shared__ unsigned long long red[DRAFT_THREADS / 64];
    const int b = blockIdx.x;
    const int32_t *h = hay + (size_t)b * hay_stride;
    const int32_t *s = needle + (size_t)b * needle_stride;
    const int hl = hay_len[b], len = needle_len[b];
    int32_t *out = out_tokens + (size_t)b * k;
    if (len < 1 || len > needle_stride || hl < 0 || hl > hay_stride) {   // device-side guard: no valid input
        for (int j = threadIdx.x; j < k; j += blockDim.x) out[j] = -1;
        if (threadIdx.x == 0) {
            if (out_match_len) out_match_len[b] = 0;
            if (out_n_copied) out_n_copied[b] = 0;
        }
        return;
    }
    unsigned long long best = 0ull;
    for (int e = threadIdx.x; e < hl; e += blockDim.x) {
        int r = 0;
        while (r <= e && r < len && (max_match <= 0 || r < max_match) && h[e - r] == s[len - 1 - r]) r++;
        if (r > 0) {
            unsigned long long key = ((unsigned long long)(uint32_t)r << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)e);
            best = key > best ? key : best;
        }
    }
    best = block_max_u64(best, red);
    const int mlen = (int)(best >> 32);
    const int e = mlen ? (int)(0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull)) : hl - 1;
    const int n_copied = mlen ? min(k, hl - 1 - e) : 0;
    for (int j = threadIdx.x; j < n_copied; j += blockDim.x) out[j] = h[e + 1 + j];
    if (threadIdx.x == 0) {
        if (out_match_len) out_match_len[b] = mlen;
        if (out_n_copied) out_n_copied[b] = n_copied;
        int32_t cur = n_copied > 0 ? h[e + n_copied] : s[len - 1];
        for (int j = n_copied; j < k; j++) {
            cur = (cur >= 0 && cur < vocab) ? next_table[cur] : -1;
            out[j] = cur;
        }
    }
}

// Bigram fit, one workgroup.  Pass 1: for every position i the pair (s[i], s[i+1]) gets the key
// (count of the pair, index of its last occurrence).  Pass 2: the last occurrence of a pair
// writes next[a] if no other pair with the same first token has a larger key.
__global__ __launch_bounds__(FIT_THREADS) void k_bigram_fit(const int32_t *__restrict__ s, int32_t n, int32_t vocab,
                                                            int32_t *__restrict__ next_table) {
    extern __shared__ unsigned long long key[];
    for (int i = threadIdx.x; i < n - 1; i += blockDim.x) {
        const int32_t a = s[i], b = s[i + 1];
        uint32_t cnt = 0, last = (uint32_t)i;
        for (int j = 0; j < n - 1; j++)
            if (s[j] == a && s[j + 1] == b) { cnt++; last = (uint32_t)j; }
        const bool ok = a >= 0 && a < vocab && b >= 0 && b < vocab;
        key[i] = ok ? (((unsigned long long)cnt << 32) | last) : 0ull;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < n - 1; i += blockDim.x) {
        const unsigned long long mine = key[i];
        if (mine == 0ull || (uint32_t)(mine & 0xFFFFFFFFull) != (uint32_t)i) continue;   // not the pair's last occurrence
        const int32_t a = s[i];
        bool best = true;
        for (int j = 0; j < n - 1; j++)
            if (s[j] == a && key[j] > mine) { best = false; break; }
        if (best) next_table[a] = s[i + 1];
    }
}

extern "C" int32_t csd_bigram_fit(const int32_t *tokens, int32_t n, int32_t vocab, int32_t *next_table, void *stream) {
    if (!tokens || !next_table) return CSD_ENULL;
    if (n < 0 || vocab < 1) return CSD_EINVAL;
    if (n > 8192) return CSD_ESHAPE;
    if (n < 2) return CSD_OK;
    hipLaunchKernelGGL(k_bigram_fit, dim3(1), dim3(FIT_THREADS), (size_t)n * sizeof(unsigned long long),
                       (hipStream_t)stream, tokens, n, vocab, next_table);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

extern "C" int32_t csd_bigram_draft(const int32_t *ctx, const int32_t *ctx_len, int32_t B, int32_t ctx_stride,
                                    const int32_t *next_table, int32_t vocab, int32_t k, int32_t max_match,
                                    int32_t *out_tokens, int32_t *out_match_len, void *stream) {
    if (!ctx || !ctx_len || !next_table) return CSD_ENULL;
    if (B < 0 || k < 0 || vocab < 1 || ctx_stride < 1) return CSD_EINVAL;
    if (k > 0 && !out_tokens) return CSD_ENULL;
    if (B == 0 || (k == 0 && !out_match_len)) return CSD_OK;   // k == 0 still reports match lengths
    hipLaunchKernelGGL(k_bigram_draft, dim3(B), dim3(DRAFT_THREADS), 0, (hipStream_t)stream, ctx, ctx_len, ctx_stride,
                       next_table, vocab, k, max_match, out_tokens, out_match_len);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

extern "C" int32_t csd_maxgram_draft(const int32_t *haystack, const int32_t *haystack_len, int32_t haystack_stride,
                                     const int32_t *needle, const int32_t *needle_len, int32_t needle_stride, int32_t B,
                                     const int32_t *next_table, int32_t vocab, int32_t k, int32_t max_match,
                                     int32_t *out_tokens, int32_t *out_match_len, int32_t *out_n_copied, void *stream) {
    if (!haystack || !haystack_len || !needle || !needle_len || !next_table) return CSD_ENULL;
    if (B < 0 || k < 0 || vocab < 1 || haystack_stride < 1 || needle_stride < 1) return CSD_EINVAL;
    if (k > 0 && !out_tokens) return CSD_ENULL;
    if (B == 0 || (k == 0 && !out_match_len && !out_n_copied)) return CSD_OK;
    hipLaunchKernelGGL(k_maxgram_enc, dim3(B), dim3(DRAFT_THREADS), 0, (hipStream_t)stream, haystack, haystack_len,
                       haystack_stride, needle, needle_len, needle_stride, next_table, vocab, k, max_match, out_tokens,
                       out_match_len, out_n_copied);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

extern "C" int32_t csd_bigram_draft_append(int32_t *ctx, int32_t ctx_stride, int32_t *ctx_len, int32_t B,
                                           const int32_t *next_table, int32_t vocab, int32_t k, int32_t max_match,
                                           const int32_t *gate, uint8_t *q_onehot_tab, const int32_t *q_base,
                                           int32_t q_stride, void *stream) {
    if (!ctx || !ctx_len || !next_table) return CSD_ENULL;
    if (B < 0 || k < 0 || vocab < 1 || ctx_stride < 1) return CSD_EINVAL;
    if (q_onehot_tab && (!q_base || q_stride < 1)) return CSD_EINVAL;
    if (B == 0) return CSD_OK;
    hipLaunchKernelGGL(k_bigram_draft_append, dim3(B), dim3(DRAFT_THREADS), 0, (hipStream_t)stream, ctx, ctx_stride, ctx_len,
                       next_table, vocab, k, max_match, gate, q_onehot_tab, q_base, q_stride);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

extern "C" int32_t csd_cascade_gate(const int32_t *ctx_len, const int32_t *loop_start, int32_t need, const int32_t *parent_gate,
                                    int32_t B, int32_t *gate, void *stream) {
    if (!ctx_len || !gate) return CSD_ENULL;
    if (B < 0) return CSD_EINVAL;
    if (B == 0) return CSD_OK;
    hipLaunchKernelGGL(k_cascade_gate, dim3((B + 63) / 64), dim3(64), 0, (hipStream_t)stream, ctx_len, loop_start, need, parent_gate,
                       B, gate);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}
