// Review forward for blocks of up to 32 rows (Section 2: one run of the reviewer scores every drafted
// position): five launches per layer, no split-K partial sums in memory, no epilogue kernels.
//
//   QKV GEMM   -> rotate q, k; q to the query buffer; K, V appended to the cache   (epilogue)
//   attention  -> key chunks in parallel, merged by the last chunk to finish
//   O GEMM     -> h += ; (h * gain) as the next GEMM's input; sum of squares per tile (epilogue)
//   gate|up    -> silu(rstd * gate) * (rstd * up) as the next GEMM's input              (epilogue)
//   down GEMM  -> h += ; (h * gain); sum of squares per tile                            (epilogue)
//
// A GEMM workgroup owns a few whole 16-feature output tiles (for one or two 16-row tiles of the block) and
// splits K over its eight waves; every wave
// streams its own K slice of the pre-tiled weights through a register ring and multiplies it with the
// activation fragments of the same slice (read from L2: no two waves need the same ones), the eight
// partial tiles are added in LDS in wave order (deterministic), and the epilogue runs in the same kernel
// on complete sums.  RMSNorm is folded around the GEMM: rmsnorm(h) * g @ W = rstd(row) * ((h * g) @ W);
// the producer of h writes h * g and one sum of squares per (row, 16-feature tile), the consumer's
// epilogue scales its output rows by 1 / sqrt(sum / d + eps).
#include <cmath>

#include "csd_internal.h"

#define CH_WAVES 8
#define CH_THREADS (CH_WAVES * 64)
#define CH_OOB ((int)0x80000000)     /* buffer offset beyond any buffer: loads give 0 and touch no memory */
#define CH_SC1 16                    /* write-through stores: the data is for workgroups on other compute dies */

enum { EPI_QKV = 0, EPI_RESID = 1, EPI_GU = 2, EPI_LOGITS = 3 };

struct ChainGemm {
    const u32x4 *Wp;          // tiles [N/16][KS][64 lanes][8 bf16]
    int KS, n_units, wbytes;  // k-steps of 32; units a workgroup owns whole (a tile; gate|up: a gate tile and its up tile)
    const bf16_t *a;          // input planes (hi, lo), fragment order (act_tiled_idx)
    int a_plane_bytes, mtp, M;
    const float *ssq_in;      // [n_ssq][ssq_rows]: sum of squares of the input's source rows per 16-feature tile (folded norm) or null
    int n_ssq, ssq_rows;      // ssq_rows: 16 * (row tiles of the call), for ssq_in and ssq_out alike
    float inv_d, eps;
    // EPI_RESID: residual stream, next norm's gain, output planes + sums of squares
    float *h;
    const float *gain;
    bf16_t *out;              // output planes (EPI_RESID, EPI_GU), fragment order
    int out_plane_bytes;
    float *ssq_out;
    int d;
    // EPI_QKV
    int m, hd, dh, layer;
    KvGeom geo;
    const int32_t *cache_len;
    const float2 *rope;       // (cos, sin) [M][dh/2] or null
    bf16_t *q;                // rotated queries, two row-major planes [..][hd]
    int q_plane_bytes;
    bf16_t *kv;
    int gelu;                 // EPI_GU: tanh-GELU instead of SiLU
    float *logits;            // EPI_LOGITS [M][V]
    int V;
};

// A buffer descriptor must sit in scalar registers.  Base addresses here are the same in every lane, but the
// compiler cannot always prove it (64-bit address arithmetic on workgroup indices may end up in vector
// registers) and then wraps every access in a loop over the distinct descriptors: say so explicitly.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t ch_rsrc(const void *p, size_t bytes) {
    const unsigned long long a = (unsigned long long)p;
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a), hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
    const int n = __builtin_amdgcn_readfirstlane((int)(bytes > 0x7FFFFFFFull ? 0x7FFFFFFFull : bytes));
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void *>(((unsigned long long)hi << 32) | lo), 0, n, 0x00020000);
}

__device__ __forceinline__ void split4(const float *v, u32x2 &hi, u32x2 &lo) {
#pragma unroll
    for (int w = 0; w < 2; w++) {
        const uint32_t hh = pack_bf16x2(v[2 * w], v[2 * w + 1]);
        hi[w] = hh;
        lo[w] = pack_bf16x2(v[2 * w] - __uint_as_float(hh << 16), v[2 * w + 1] - __uint_as_float(hh & 0xFFFF0000u));
    }
}

// Four consecutive columns of one row into the two planes of a fragment-ordered activation buffer.
__device__ __forceinline__ void store_planes4(bf16_t *out, int plane_bytes, int mtp, int row, int col, const float *v) {
    u32x2 hi, lo;
    split4(v, hi, lo);
    const int off = (int)(act_tiled_idx(row, col, mtp) * 2);
    const __amdgpu_buffer_rsrc_t r = ch_rsrc(out, (size_t)2 * plane_bytes);
    __builtin_amdgcn_raw_buffer_store_b64(hi, r, off, 0, CH_SC1);
    __builtin_amdgcn_raw_buffer_store_b64(lo, r, off + plane_bytes, 0, CH_SC1);
}

// This wave's share of a GEMM: the workgroup's tiles [t0, t0 + nt) (nt <= NT), the wave's k-steps [ks0, ks1).
struct GemmShare {
    int t0, nt, ks0, ks1;
};
template <int EPI>
__device__ __forceinline__ GemmShare gemm_share(const ChainGemm &P, int wg, int G, int w) {
    constexpr int UT = EPI == EPI_GU ? 2 : 1;
    // Workgroups go to the eight compute dies round-robin, and what a die can pull from memory is what bounds the
    // launch: the units are dealt so that every die gets the same number (consecutive shares to the workgroups of one
    // die), not merely every workgroup within one of the next (688 units over 256 workgroups gave three dies 96 units
    // and five dies 80, and the launch lasted as long as the dies with 96).
    if (G % 8 == 0) wg = (wg & 7) * (G >> 3) + (wg >> 3);
    const int u0 = (int)((long long)P.n_units * wg / G), u1 = (int)((long long)P.n_units * (wg + 1) / G);
    return GemmShare{u0 * UT, (u1 - u0) * UT, P.KS * w / CH_WAVES, P.KS * (w + 1) / CH_WAVES};
}

// Every load of the GEMM is issued unconditionally (what must not be read gets an offset beyond the buffer),
// so the compiler can count the loads in flight and wait for exactly the oldest.
template <int NT>
__device__ __forceinline__ void gemm_load_w(u32x4 (&W)[NT], const ChainGemm &P, const GemmShare &S, __amdgpu_buffer_rsrc_t rw, int ks,
                                            int lane) {
    const bool in = ks < S.ks1;   // uniform
#pragma unroll
    for (int j = 0; j < NT; j++) {
        const bool tv = in && j < S.nt;
        W[j] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rw, tv ? lane * 16 : CH_OOB,
                                                                              tv ? ((S.t0 + j) * P.KS + ks) * 1024 : 0, 2));
    }
}
template <int MT>
__device__ __forceinline__ void gemm_load_a(u32x4 (&A)[MT][2], const ChainGemm &P, const GemmShare &S, __amdgpu_buffer_rsrc_t ra, int ks,
                                            const int (&voff_a)[MT]) {
    const bool in = ks < S.ks1;   // uniform
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        A[mt][0] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(ra, in ? voff_a[mt] : CH_OOB,
                                                                                  in ? (ks * P.mtp + mt) * 1024 : 0, 0));
        A[mt][1] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                                 ra, in ? voff_a[mt] : CH_OOB, in ? P.a_plane_bytes + (ks * P.mtp + mt) * 1024 : 0, 0));
    }
}

// The first R k-steps of a wave's weight stream: they depend on nothing the other workgroups produce, so a
// kernel that runs several GEMMs may issue them before the device-wide barrier in front of the GEMM.
template <int NT, int R>
__device__ __forceinline__ void gemm_prefetch(u32x4 (&Wr)[R][NT], const ChainGemm &P, const GemmShare &S) {
    const __amdgpu_buffer_rsrc_t rw = ch_rsrc(P.Wp, (size_t)P.wbytes);
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int r = 0; r < R; r++) gemm_load_w<NT>(Wr[r], P, S, rw, S.ks0 + r, lane);
}

// What the epilogue of one (tile, row tile) needs besides the sums, fetched before the main loop.
struct EpiIn {
    f32x4 hcur, gcur;
    float2 cs[4];
    int pos;
};

// The epilogue of one output tile (gate|up: a gate tile and its up tile) for the 16 rows of one row tile, on complete,
// rstd-scaled sums v.  row: this lane's block row; T: global index of the (first) tile.  No workgroup barrier inside.
template <int EPI>
__device__ __forceinline__ void gemm_epilogue(const ChainGemm &P, const f32x4 *v, const EpiIn &E, int row, int T, int g) {
    constexpr int UT = EPI == EPI_GU ? 2 : 1;
    const bool valid = row < P.M;
    if (EPI == EPI_RESID) {
        const f32x4 hv = E.hcur + v[0];
        float ss = hv[0] * hv[0] + hv[1] * hv[1] + hv[2] * hv[2] + hv[3] * hv[3];
        ss += __shfl_xor(ss, 16, 64);
        ss += __shfl_xor(ss, 32, 64);
        if (!valid) return;
        const int col = T * 16 + 4 * g;
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, hv), ch_rsrc(P.h, (size_t)P.M * P.d * 4),
                                               (int)(((size_t)row * P.d + col) * 4), 0, CH_SC1);
        const float o[4] = {hv[0] * E.gcur[0], hv[1] * E.gcur[1], hv[2] * E.gcur[2], hv[3] * E.gcur[3]};
        store_planes4(P.out, P.out_plane_bytes, P.mtp, row, col, o);
        if (g == 0)
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, ss),
                                                  ch_rsrc(P.ssq_out, (size_t)(P.d / 16) * P.ssq_rows * 4), (T * P.ssq_rows + row) * 4, 0, CH_SC1);
    } else if (EPI == EPI_GU) {
        if (!valid) return;
        float o[4];
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const float gt = v[0][r], up = v[UT - 1][r];
            const float a = P.gelu ? 0.5f * gt * (1.0f + tanhf(0.7978845608028654f * (gt + 0.044715f * gt * gt * gt)))
                                   : gt / (1.0f + expf(-gt));
            o[r] = a * up;
        }
        store_planes4(P.out, P.out_plane_bytes, P.mtp, row, (T / 2) * 16 + 4 * g, o);
    } else if (EPI == EPI_LOGITS) {
        if (!valid) return;
        *reinterpret_cast<f32x4 *>(P.logits + (size_t)row * P.V + T * 16 + 4 * g) = v[0];
    } else {   // EPI_QKV
        const int tiles_per_region = P.hd / 16, tiles_per_head = P.dh / 16;
        const int region = T / tiles_per_region, tr = T % tiles_per_region;
        const int head = tr / tiles_per_head, ti = tr % tiles_per_head;
        const int b = valid ? row / P.m : 0;
        const int pos = E.pos;
        if (region < 2) {
            // tiles of q and k hold whole rotary pairs: lane groups 0, 1 the first-half entries 8 ti .. 8 ti + 7,
            // groups 2, 3 their partners; one exchange across the wave brings the pair together
            float o[4];
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const float other = __shfl_xor(v[0][r], 32, 64);
                const float c = E.cs[r].x, s = E.cs[r].y;
                o[r] = g < 2 ? v[0][r] * c - other * s : other * s + v[0][r] * c;
            }
            if (!valid) return;
            const int p0 = 16 * ti + 4 * g;                    // place inside the head, pair order
            if (region == 0) {
                u32x2 hi, lo;
                split4(o, hi, lo);
                const __amdgpu_buffer_rsrc_t rq = ch_rsrc(P.q, (size_t)2 * P.q_plane_bytes);
                const int off = (int)(((size_t)row * P.hd + head * P.dh + p0) * 2);
                __builtin_amdgcn_raw_buffer_store_b64(hi, rq, off, 0, CH_SC1);
                __builtin_amdgcn_raw_buffer_store_b64(lo, rq, off + P.q_plane_bytes, 0, CH_SC1);
            } else if (pos >= 0 && pos < P.geo.seq_pad) {
                u32x2 kk;
                kk[0] = pack_bf16x2(o[0], o[1]);
                kk[1] = pack_bf16x2(o[2], o[3]);
                // (the sequence, hence the head's region, differs from lane to lane: one descriptor for the layer's
                // keys, the rest in the per-lane offset; written through, the attention step may run on another die)
                const size_t he = kv_head_elems(P.geo);
                __builtin_amdgcn_raw_buffer_store_b64(kk, ch_rsrc(P.kv + kv_k_off(P.geo, P.layer, 0, 0), (size_t)P.geo.Bmax * P.geo.H * he * 2),
                                                      (int)((((size_t)b * P.geo.H + head) * he + (size_t)pos * P.dh + p0) * 2), 0, CH_SC1);
            }
        } else if (valid && pos >= 0 && pos < P.geo.seq_pad) {
            const size_t he = kv_head_elems(P.geo);
            const __amdgpu_buffer_rsrc_t rv = ch_rsrc(P.kv + kv_v_off(P.geo, P.layer, 0, 0), (size_t)P.geo.Bmax * P.geo.H * he * 2);
#pragma unroll
            for (int r = 0; r < 4; r++)
                __builtin_amdgcn_raw_buffer_store_b16(f32_to_bf16(v[0][r]), rv,
                                                      (int)((((size_t)b * P.geo.H + head) * he + kv_v_idx(P.geo, 16 * ti + 4 * g + r, pos)) * 2), 0,
                                                      CH_SC1);
        }
    }
}

// The GEMM of one workgroup after gemm_prefetch: the wave's k-steps through the rings for MT row tiles of 16 rows, the
// eight partial tiles added in LDS in wave order (one row tile at a time), the epilogue.  LDS: red [8 waves][NT][64 lanes]
// 16-byte words, then [8 waves][16 MT rows] floats.  Every wave of the workgroup must call it (it holds workgroup barriers).
template <int NT, int R, int EPI, int MT>
__device__ __forceinline__ void gemm_run(u32x4 (&Wr)[R][NT], const ChainGemm &P, const GemmShare &S, char *smem) {
    f32x4 *red = reinterpret_cast<f32x4 *>(smem);
    float *rs_part = reinterpret_cast<float *>(smem + (size_t)CH_WAVES * NT * 64 * 16);
    constexpr int UT = EPI == EPI_GU ? 2 : 1;
    const int lane = threadIdx.x & 63, t = lane & 15, g = lane >> 4;
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int t0 = S.t0, nt = S.nt, ks0 = S.ks0, ks1 = S.ks1;
    const __amdgpu_buffer_rsrc_t rw = ch_rsrc(P.Wp, (size_t)P.wbytes);
    const __amdgpu_buffer_rsrc_t ra = ch_rsrc(P.a, (size_t)2 * P.a_plane_bytes);
    int voff_a[MT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) voff_a[mt] = mt * 16 + t < P.M ? (4 * t + g) * 16 : CH_OOB;

    // partial sums of squares of the rows behind the folded norm: wave w, lane group g take every 32nd tile.
    // Eight independent loads per row tile and turn (a dependent chain of them would hold up the rings behind it).
    float ssq[MT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) ssq[mt] = 0.f;
    if (P.ssq_in) {
        const __amdgpu_buffer_rsrc_t rq = ch_rsrc(P.ssq_in, (size_t)P.n_ssq * P.ssq_rows * 4);
        for (int base = 0; base < P.n_ssq; base += 8 * 4 * CH_WAVES) {
            float sv[MT][8];
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
#pragma unroll
                for (int n = 0; n < 8; n++) {
                    const int i = base + n * 4 * CH_WAVES + w * 4 + g;
                    sv[mt][n] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                                              rq, i < P.n_ssq ? (i * P.ssq_rows + mt * 16 + t) * 4 : CH_OOB, 0, 0));
                }
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
#pragma unroll
                for (int n = 0; n < 8; n++) ssq[mt] += sv[mt][n];
        }
    }
    u32x4 Ar[R][MT][2];
    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int j = 0; j < NT; j++) acc[mt][j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < R; r++) gemm_load_a<MT>(Ar[r], P, S, ra, ks0 + r, voff_a);

    // epilogue inputs that do not depend on the sums: fetched now, used after the reduction
    EpiIn E[MT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        const int row = mt * 16 + t;
        E[mt].hcur = E[mt].gcur = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < 4; r++) E[mt].cs[r] = float2{1.f, 0.f};
        E[mt].pos = -1;
        if (EPI == EPI_RESID && w < nt && row < P.M) {
            const int col = (t0 + w) * 16 + 4 * g;
            E[mt].hcur = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(ch_rsrc(P.h, (size_t)P.M * P.d * 4),
                                                                                        (int)(((size_t)row * P.d + col) * 4), 0, 0));
            E[mt].gcur = *reinterpret_cast<const f32x4 *>(P.gain + col);
        }
        if (EPI == EPI_QKV && w < nt && row < P.M) {
            const int ti = ((t0 + w) % (P.hd / 16)) % (P.dh / 16);
            E[mt].pos = P.cache_len[row / P.m] + row % P.m;
            if (P.rope && (t0 + w) < 2 * (P.hd / 16)) {
#pragma unroll
                for (int r = 0; r < 4; r++) E[mt].cs[r] = P.rope[(size_t)row * (P.dh / 2) + 8 * ti + 4 * (g & 1) + r];
            }
        }
    }
    if (P.ssq_in) {
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            float s = ssq[mt];
            s += __shfl_xor(s, 16, 64);
            s += __shfl_xor(s, 32, 64);
            if (g == 0) rs_part[(w * MT + mt) * 16 + t] = s;
        }
    }

    for (int ks = ks0; ks < ks1; ks += R) {
#pragma unroll
        for (int r = 0; r < R; r++) {
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
#pragma unroll
                for (int j = 0; j < NT; j++)
                    acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, Wr[r][j]),
                                                                         __builtin_bit_cast(bf16x8, Ar[r][mt][0]), acc[mt][j], 0, 0, 0);
#pragma unroll
                for (int j = 0; j < NT; j++)
                    acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, Wr[r][j]),
                                                                         __builtin_bit_cast(bf16x8, Ar[r][mt][1]), acc[mt][j], 0, 0, 0);
            }
            gemm_load_w<NT>(Wr[r], P, S, rw, ks + r + R, lane);
            gemm_load_a<MT>(Ar[r], P, S, ra, ks + r + R, voff_a);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // ------------------------------------------------------------------ reduction and epilogue, a row tile at a time:
    // wave e takes unit e
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        if (mt > 0) __syncthreads();                           // the sums of the row tile before have been read
#pragma unroll
        for (int j = 0; j < NT; j++) red[(w * NT + j) * 64 + lane] = acc[mt][j];
        __syncthreads();
        if (w * UT < nt) {
            float rstd = 1.f;
            if (P.ssq_in) {
                float s = 0.f;
#pragma unroll
                for (int i = 0; i < CH_WAVES; i++) s += rs_part[(i * MT + mt) * 16 + t];
                rstd = rsqrtf(s * P.inv_d + P.eps);
            }
            f32x4 v[UT];
#pragma unroll
            for (int x = 0; x < UT; x++) {
                v[x] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int i = 0; i < CH_WAVES; i++) v[x] += red[(i * NT + w * UT + x) * 64 + lane];
                v[x] *= rstd;
            }
            gemm_epilogue<EPI>(P, v, E[mt], mt * 16 + t, t0 + w * UT, g);
        }
    }
}

template <int NT, int R, int EPI, int MT>
__global__ __launch_bounds__(CH_THREADS) void kc_gemm(const ChainGemm P) {
    extern __shared__ __align__(16) char ch_smem[];
    const GemmShare S = gemm_share<EPI>(P, blockIdx.x, gridDim.x, __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)));
    u32x4 Wr[R][NT];
    gemm_prefetch<NT, R>(Wr, P, S);
    gemm_run<NT, R, EPI, MT>(Wr, P, S, ch_smem);
}

// Causal attention of a block of up to 16 rows over the cached prefix, one launch per layer.  A workgroup
// of four waves takes 128 keys of one (sequence, head): each wave one 32-key tile with both products on the
// matrix cores, transposed so that no operand passes through LDS (S^T = K q^T, O^T = V^T P^T; V is cached
// transposed), the four softmax states are merged in LDS, and the workgroup writes one partial state per
// chunk.  The last workgroup of a (sequence, head) to finish (an arrival counter) merges the chunks and
// writes the rows as the O projection's input; the counter is back at zero when the kernel ends.
#define CA_KEYS 128
#define CA_MAX_CHUNKS 128     /* the merge keeps a weight per (chunk, row) in LDS: sequences of up to 16384 cached rows */
struct AttnArgs {
    const bf16_t *q;          // rotated queries, two row-major planes [..][hd]
    int q_plane, m;
    const int32_t *cache_len;
    KvGeom geo;
    int layer;
    const bf16_t *kv;
    float scale;
    float *part;              // chunk states [B][H][chunks_max][16 rows][DH + 4]
    int chunks_max;
    unsigned *counters;       // arrivals per (sequence, head): zero between launches
    const unsigned long long *anc;   // tree block: per block row the rows it sees (see AttnMode), or null
    const float *bias_hd;     // arch 1 self-attention: [H][128] bias by distance query - key (127: that or more), or null
    int fixed_nk;             // > 0 (arch 1 cross-attention): every row sees keys [0, fixed_nk), whatever cache_len says
    bf16_t *out;              // merged rows: the O projection's input planes, fragment order
    int out_plane_bytes, mtp;
};
template <int DH>
struct AttnLds {
    f32x4 o[4][DH / 16][64];
    float m[4][16], l[4][16];
    float mc[CA_MAX_CHUNKS * 16], lc[CA_MAX_CHUNKS * 16], w[CA_MAX_CHUNKS * 16];   // chunk states and weights of the merge
    unsigned old;
    unsigned pad[3];
};

// One chunk of one (sequence, head) by a group of four waves (gtid = thread index in the group, 0 .. 255).
// Holds five workgroup barriers whatever `have` says, so groups with and without an item stay in step.
template <int DH>
__device__ __forceinline__ void attn_item(const AttnArgs &A, AttnLds<DH> &L, bool have, int c, int hh, int b, int gtid) {
    constexpr int PS = DH + 4;                               // floats per partial row: DH outputs, max, sum, pad
    constexpr int DT = DH / 16;
    const KvGeom &geo = A.geo;
    const int m = A.m;
    const int lane = gtid & 63, col = lane & 15, g = lane >> 4;
    const int wv = __builtin_amdgcn_readfirstlane(gtid >> 6);
    const int hd = geo.H * DH;
    const int kb = c * CA_KEYS + wv * 32;                    // this wave's 32 keys
    // Every load is issued before the cached length is known (their addresses do not depend on it; rows past
    // the end are masked below, rows past the cache are outside the buffer and read as zeros).
    const size_t head_bytes = have ? kv_head_elems(geo) * 2 : 0;
    const __amdgpu_buffer_rsrc_t rk = ch_rsrc(A.kv + kv_k_off(geo, A.layer, b, hh), head_bytes);
    const __amdgpu_buffer_rsrc_t rv = ch_rsrc(A.kv + kv_v_off(geo, A.layer, b, hh), head_bytes);
    const __amdgpu_buffer_rsrc_t rqb = ch_rsrc(A.q, have ? (size_t)4 * A.q_plane : 0);
    u32x4 qf[DH / 32][2], kf[2][DH / 32], vf[DT];
#pragma unroll
    for (int s = 0; s < DH / 32; s++) {
        const int qo = col < m ? (int)(((size_t)(b * m + col) * hd + hh * DH + s * 32 + 8 * g) * 2) : CH_OOB;
        qf[s][0] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rqb, qo, 0, 0));
        qf[s][1] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rqb, qo, A.q_plane * 2, 0));
    }
    // A operands.  K: A-row r of tile T is key kb + 8 (r / 4) + 4 T + r % 4, so lane group g ends up with the
    // scores of keys kb + 8 g .. + 7; V^T: row = feature dt * 16 + col, 8 consecutive keys per lane.
#pragma unroll
    for (int T = 0; T < 2; T++) {
        const int key = kb + 8 * (col >> 2) + 4 * T + (col & 3);
#pragma unroll
        for (int s = 0; s < DH / 32; s++)
            kf[T][s] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rk, (key * DH + 8 * g + s * 32) * 2, 0, 0));
    }
#pragma unroll
    for (int dt = 0; dt < DT; dt++)
        vf[dt] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rv, (int)(kv_v_idx(geo, dt * 16 + col, kb + 8 * g) * 2), 0, 0));
    const bool causal = A.fixed_nk <= 0;
    const int t = (have && causal) ? A.cache_len[b] : 0;
    const int nk = max(0, min(causal ? t + m : A.fixed_nk, geo.seq_pad));   // cache rows in play for this block
    const int nch = (nk + CA_KEYS - 1) / CA_KEYS;
    const bool active = have && c < nch;                     // a chunk past the end is not counted
    const int qpos = t + col;                                // block row `col` sees cache rows 0 .. qpos
    const unsigned long long anc_row = (A.anc && have && col < m) ? A.anc[b * m + col] : 0ull;
    float bias[8];                                           // requested ahead of the scores they are added to
#pragma unroll
    for (int j = 0; j < 8; j++) {
        const int dist = qpos - (kb + 8 * g + j);
        bias[j] = (A.bias_hd && have && dist >= 0) ? A.bias_hd[hh * 128 + min(dist, 127)] : 0.f;
    }
    float mrun = -INFINITY, lrun = 0.f;
    f32x4 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; dt++) oacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (active && kb < nk) {                                 // uniform over the wave
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
        float sv[8], mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const int key = kb + 8 * g + j;
            const bool seen = (A.anc ? tree_sees(anc_row, key, t) : (!causal || key <= qpos)) && key < nk;
            sv[j] = seen ? sT[j >> 2][j & 3] * A.scale + bias[j] : -INFINITY;
            mx = fmaxf(mx, sv[j]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        float pv[8], psum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; j++) {
            pv[j] = (sv[j] == -INFINITY) ? 0.f : expf(sv[j] - mx);
            psum += pv[j];
        }
        psum += __shfl_xor(psum, 16, 64);
        psum += __shfl_xor(psum, 32, 64);
        mrun = mx;
        lrun = psum;
        u32x4 pf, pl;                                        // hi and lo planes of the probabilities
#pragma unroll
        for (int w2 = 0; w2 < 4; w2++) {
            const uint32_t hpk = pack_bf16x2(pv[2 * w2], pv[2 * w2 + 1]);
            pf[w2] = hpk;
            pl[w2] = pack_bf16x2(pv[2 * w2] - __uint_as_float(hpk << 16), pv[2 * w2 + 1] - __uint_as_float(hpk & 0xFFFF0000u));
        }
        const bool tail = kb + 32 > nk;                      // rows past nk may hold anything: zero them
#pragma unroll
        for (int dt = 0; dt < DT; dt++) {
            u32x4 v = vf[dt];
            if (tail) {
#pragma unroll
                for (int w2 = 0; w2 < 4; w2++) {
                    const int k0 = kb + 8 * g + 2 * w2;
                    v[w2] &= (k0 < nk ? 0x0000FFFFu : 0u) | (k0 + 1 < nk ? 0xFFFF0000u : 0u);
                }
            }
            oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v), __builtin_bit_cast(bf16x8, pf), oacc[dt], 0, 0, 0);
            oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v), __builtin_bit_cast(bf16x8, pl), oacc[dt], 0, 0, 0);
        }
    }
    // ---- the four tiles of the chunk, merged in LDS; wave wv writes output tiles wv, wv + 4, ...
#pragma unroll
    for (int dt = 0; dt < DT; dt++) L.o[wv][dt][lane] = oacc[dt];
    if (g == 0) {
        L.m[wv][col] = mrun;
        L.l[wv][col] = lrun;
    }
    __syncthreads();
    if (active) {
        float mstar = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; i++) mstar = fmaxf(mstar, L.m[i][col]);
        float wgt[4], lsum = 0.f;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            wgt[i] = L.m[i][col] == -INFINITY ? 0.f : expf(L.m[i][col] - mstar);
            lsum += wgt[i] * L.l[i][col];
        }
        float *po = A.part + (((size_t)b * geo.H + hh) * A.chunks_max + c) * 16 * PS;
        const __amdgpu_buffer_rsrc_t rp = ch_rsrc(po, (size_t)16 * PS * 4);
        for (int dt = wv; dt < DT; dt += 4) {
            f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < 4; i++) o += L.o[i][dt][lane] * wgt[i];
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, o), rp, (col * PS + dt * 16 + 4 * g) * 4, 0, CH_SC1);
        }
        if (wv == 0 && g == 0) {
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, mstar), rp, (col * PS + DH) * 4, 0, CH_SC1);
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, lsum), rp, (col * PS + DH + 1) * 4, 0, CH_SC1);
        }
    }
    // ---- arrival: the stores above are acknowledged before the counter moves
    __builtin_amdgcn_s_waitcnt(0x0F70);                      // vmcnt(0)
    __syncthreads();
    unsigned *cnt = A.counters + b * geo.H + hh;
    if (gtid == 0) L.old = active ? __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0xFFFFFFFFu;
    __syncthreads();
    // ---- last to arrive: merge the chunk states of this (sequence, head).  They were written through to memory,
    // and this compute die's L2 (emptied when the kernel started) cannot hold an older copy of them.
    const bool last = active && L.old == (unsigned)(nch - 1);
    const float *pbase = A.part + ((size_t)b * geo.H + hh) * A.chunks_max * 16 * PS;
    const __amdgpu_buffer_rsrc_t rm = ch_rsrc(pbase, last ? (size_t)A.chunks_max * 16 * PS * 4 : 0);
    // out[r][x] = sum_c weight[c][r] * acc_c[r][x] with weight[c][r] = e^(m_c - m*) / sum_c l_c e^(m_c - m*).  A thread
    // takes feature x of every (256 / DH)-th row; the accumulators of four rows x sixteen chunks are requested
    // together, and the first such batch before the states, so that the common case is one memory round trip.
    const int x = gtid % DH;
    constexpr int RG = 256 / DH;
    const int r_first = gtid / DH;
    float ac[4][16];
#define CA_LOAD_ACC(R0, C0)                                                                                          \
    _Pragma("unroll") for (int rr = 0; rr < 4; rr++) _Pragma("unroll") for (int u = 0; u < 16; u++) {                \
        const int r_ = (R0) + rr * RG; /* (the scalar offset operand must be uniform: the per-thread part is the vector offset) */ \
        ac[rr][u] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(                                  \
                                                  rm, (r_ < m && (C0) + u < nch) ? ((((C0) + u) * 16 + r_) * PS + x) * 4 : CH_OOB, 0, 0)); \
    }
    if (last) {
        CA_LOAD_ACC(r_first, 0)
        const int r = gtid & 15;
        for (int cc = gtid >> 4; cc < nch; cc += 16) {
            const int o = (cc * 16 + r) * PS * 4;
            L.mc[cc * 16 + r] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rm, o, DH * 4, 0));
            L.lc[cc * 16 + r] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rm, o, (DH + 1) * 4, 0));
        }
    }
    __syncthreads();
    if (last) {
        const int r = gtid & 15;
        float mst = -INFINITY;
        for (int cc = 0; cc < nch; cc++) mst = fmaxf(mst, L.mc[cc * 16 + r]);
        float den = 0.f;
        for (int cc = 0; cc < nch; cc++) {
            const float mc = L.mc[cc * 16 + r];
            den += (mc == -INFINITY ? 0.f : expf(mc - mst)) * L.lc[cc * 16 + r];       // chunks in order
        }
        const float inv = den > 0.f ? 1.0f / den : 0.f;
        for (int cc = gtid >> 4; cc < nch; cc += 16) {
            const float mc = L.mc[cc * 16 + r];
            L.w[cc * 16 + r] = (mc == -INFINITY ? 0.f : expf(mc - mst)) * inv;
        }
    }
    __syncthreads();
    if (last) {
        const __amdgpu_buffer_rsrc_t ro = ch_rsrc(A.out, (size_t)2 * A.out_plane_bytes);
        for (int r0 = r_first; r0 < m; r0 += 4 * RG) {
            float num[4] = {0.f, 0.f, 0.f, 0.f};
            for (int c0 = 0; c0 < nch; c0 += 16) {
                if (r0 != r_first || c0 != 0) CA_LOAD_ACC(r0, c0)
#pragma unroll
                for (int rr = 0; rr < 4; rr++)
#pragma unroll
                    for (int u = 0; u < 16; u++)
                        if (r0 + rr * RG < m && c0 + u < nch) num[rr] += ac[rr][u] * L.w[(c0 + u) * 16 + r0 + rr * RG];
            }
#pragma unroll
            for (int rr = 0; rr < 4; rr++) {
                const int r = r0 + rr * RG;
                if (r >= m) break;
                const bf16_t hi = f32_to_bf16(num[rr]);
                const int off = (int)(act_tiled_idx(b * m + r, hh * DH + x, A.mtp) * 2);
                __builtin_amdgcn_raw_buffer_store_b16(hi, ro, off, 0, CH_SC1);
                __builtin_amdgcn_raw_buffer_store_b16(f32_to_bf16(num[rr] - bf16_to_f32(hi)), ro, off + A.out_plane_bytes, 0, CH_SC1);
            }
        }
        if (gtid == 0) __hip_atomic_store(cnt, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
#undef CA_LOAD_ACC
}

// Causal attention of a block of up to 16 rows over the cached prefix, one launch per layer.  A workgroup
// of four waves takes 128 keys of one (sequence, head): each wave one 32-key tile with both products on the
// matrix cores, transposed so that no operand passes through LDS (S^T = K q^T, O^T = V^T P^T; V is cached
// transposed), the four softmax states are merged in LDS, and the workgroup writes one partial state per
// chunk.  The last workgroup of a (sequence, head) to finish (an arrival counter) merges the chunks and
// writes the rows as the O projection's input; the counter is back at zero when the kernel ends.
template <int DH>
__global__ __launch_bounds__(256) void kc_attn(const AttnArgs A) {
    __shared__ __align__(16) AttnLds<DH> L;
    // Grid (head, sequence, chunk): the last chunk of a head holds little besides the block's own rows, and with the chunk
    // index slowest those short workgroups are dispatched after every long one has a compute unit of its own.
    attn_item<DH>(A, L, true, blockIdx.z, blockIdx.x, blockIdx.y, threadIdx.x);
}

// h[r] = E[token[r]]; (h * gain) as the first GEMM's input, the sums of squares per 16-feature tile, and the
// rotary table of the call's positions.  One workgroup per block row, one thread per 16-feature tile.
__global__ __launch_bounds__(256) void kc_embed(const int32_t *__restrict__ tokens, const bf16_t *__restrict__ E, int V, int d,
                                                const float *__restrict__ gain, float *__restrict__ h, bf16_t *__restrict__ out,
                                                int out_plane_bytes, int mtp, float *__restrict__ ssq_out,
                                                int ssq_rows, const int32_t *__restrict__ cache_len, int m, int dh, float theta,
                                                float2 *__restrict__ rope, const int32_t *__restrict__ depth) {
    const int r = blockIdx.x;
    const int tok = tokens[r];
    const bool ok = tok >= 0 && tok < V;
    for (int T = threadIdx.x; T < d / 16; T += blockDim.x) {
        float ss = 0.f;
#pragma unroll
        for (int c4 = 0; c4 < 4; c4++) {
            const int col = T * 16 + c4 * 4;
            u32x2 e = u32x2{0u, 0u};
            if (ok) e = *reinterpret_cast<const u32x2 *>(E + (size_t)tok * d + col);
            const f32x4 hv = f32x4{__uint_as_float(e[0] << 16), __uint_as_float(e[0] & 0xFFFF0000u), __uint_as_float(e[1] << 16),
                                   __uint_as_float(e[1] & 0xFFFF0000u)};
            *reinterpret_cast<f32x4 *>(h + (size_t)r * d + col) = hv;
            const f32x4 gv = *reinterpret_cast<const f32x4 *>(gain + col);
            const float o[4] = {hv[0] * gv[0], hv[1] * gv[1], hv[2] * gv[2], hv[3] * gv[3]};
            store_planes4(out, out_plane_bytes, mtp, r, col, o);
            ss += (hv[0] * hv[0] + hv[1] * hv[1]) + (hv[2] * hv[2] + hv[3] * hv[3]);
        }
        ssq_out[T * ssq_rows + r] = ss;
    }
    if (theta > 0.f) {
        // the position of a row: where it sits in a plain block, how far it is from row 0 in a tree block
        const int pos = cache_len[r / m] + (depth ? depth[r] : r % m), half = dh / 2;
        for (int x = threadIdx.x; x < half; x += blockDim.x) {
            const double ang = (double)pos * pow((double)theta, -2.0 * (double)x / (double)dh);
            rope[(size_t)r * half + x] = float2{(float)cos(ang), (float)sin(ang)};
        }
    }
}

// ------------------------------------------------------------------------------- host driver

#define CH_MT_MAX 2          /* row tiles of 16 rows a launch covers: blocks of up to 32 rows */

template <int NT, int R, int EPI, int MT>
static hipError_t chain_allow_lds() {
    return hipFuncSetAttribute((const void *)kc_gemm<NT, R, EPI, MT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               CH_WAVES * NT * 64 * 16 + CH_WAVES * MT * 16 * 4);
}

#ifndef CH_R1
#define CH_R1 4
#endif
// (tiles per workgroup, ring depth): one row tile; and two row tiles, where the accumulators and the
// activation ring take more registers and the rings are shallower
#define CH_FOR_ALL_NT(X, EPI, MT) X(1, CH_R1, EPI, MT) X(2, 6, EPI, MT) X(3, 4, EPI, MT) X(4, 4, EPI, MT) X(6, 2, EPI, MT) X(8, 2, EPI, MT)
#define CH_FOR_ALL_NT_TALL(X, EPI, MT) X(1, 4, EPI, MT) X(2, 3, EPI, MT) X(3, 2, EPI, MT) X(4, 2, EPI, MT) X(6, 2, EPI, MT) X(8, 2, EPI, MT)
// (the QKV epilogue holds the most state: eight tiles with two row tiles do not fit the registers, and a model
// whose QKV matrix has more than 6 * 256 column tiles takes the per-operation kernels for such blocks)
#define CH_FOR_QKV_TALL(X, MT) X(1, 4, EPI_QKV, MT) X(2, 3, EPI_QKV, MT) X(3, 2, EPI_QKV, MT) X(4, 2, EPI_QKV, MT) X(6, 2, EPI_QKV, MT)
#define CH_FOR_GU(X, MT) X(2, 6, EPI_GU, MT) X(4, 4, EPI_GU, MT) X(6, 2, EPI_GU, MT) X(8, 2, EPI_GU, MT)
#define CH_FOR_GU_TALL(X, MT) X(2, 3, EPI_GU, MT) X(4, 2, EPI_GU, MT) X(6, 2, EPI_GU, MT) X(8, 2, EPI_GU, MT)

int32_t csd_chain_setup() {
#define CH_ALLOW(NT, R, EPI, MT) CSD_HIP((chain_allow_lds<NT, R, EPI, MT>()));
    CH_FOR_ALL_NT(CH_ALLOW, EPI_QKV, 1)
    CH_FOR_ALL_NT(CH_ALLOW, EPI_RESID, 1)
    CH_FOR_ALL_NT(CH_ALLOW, EPI_LOGITS, 1)
    CH_FOR_GU(CH_ALLOW, 1)
    CH_FOR_QKV_TALL(CH_ALLOW, 2)
    CH_FOR_ALL_NT_TALL(CH_ALLOW, EPI_RESID, 2)
    CH_FOR_ALL_NT_TALL(CH_ALLOW, EPI_LOGITS, 2)
    CH_FOR_GU_TALL(CH_ALLOW, 2)
#undef CH_ALLOW
    return CSD_OK;
}

template <int EPI, int MT>
static int32_t chain_launch_mt(ChainGemm &P, int G, int per, hipStream_t st) {
#define CH_LAUNCH(NT, R, E, MT_)                                                                                   \
    if (per <= NT) {                                                                                              \
        hipLaunchKernelGGL((kc_gemm<NT, R, E, MT_>), dim3(G), dim3(CH_THREADS),                                    \
                           CH_WAVES * NT * 64 * 16 + CH_WAVES * MT_ * 16 * 4, st, P);                              \
        return CSD_OK;                                                                                            \
    }
    if constexpr (MT == 1) {
        if constexpr (EPI == EPI_GU) {
            CH_FOR_GU(CH_LAUNCH, MT)
        } else {
            CH_FOR_ALL_NT(CH_LAUNCH, EPI, MT)
        }
    } else {
        if constexpr (EPI == EPI_GU) {
            CH_FOR_GU_TALL(CH_LAUNCH, MT)
        } else if constexpr (EPI == EPI_QKV) {
            CH_FOR_QKV_TALL(CH_LAUNCH, MT)
        } else {
            CH_FOR_ALL_NT_TALL(CH_LAUNCH, EPI, MT)
        }
    }
#undef CH_LAUNCH
    return CSD_ESHAPE;
}

template <int EPI>
static int32_t chain_launch(ChainGemm &P, int n_tiles, hipStream_t st) {
    constexpr int UT = EPI == EPI_GU ? 2 : 1;
    P.n_units = n_tiles / UT;
    // a workgroup per compute unit, or as many more as keep a workgroup's tiles to eight
    int G = P.n_units < 256 ? P.n_units : 256;
    if ((P.n_units + G - 1) / G * UT > 8) G = (P.n_units * UT + 7) / 8;
    const int per = (P.n_units + G - 1) / G * UT;            // most tiles of a workgroup
    const int mt = (P.M + 15) / 16;
    if (mt == 1) return chain_launch_mt<EPI, 1>(P, G, per, st);
    if (mt == 2) return chain_launch_mt<EPI, 2>(P, G, per, st);
    return CSD_ESHAPE;
}

bool csd_chain_eligible(const csd_model *mod, int32_t B, int32_t m) {
    // (the cache appends address a layer's keys, or values, through one 32-bit offset)
    const size_t layer_kv = (size_t)mod->cfg.max_batch * mod->cfg.n_heads * mod->seq_pad * mod->cfg.head_dim * 2;
    if (B * m > 16 && 3 * mod->hd / 16 > 6 * 256) return false;
    return mod->chain_on && B * m <= 16 * CH_MT_MAX && mod->seq_pad <= CA_KEYS * CA_MAX_CHUNKS && layer_kv < (1ull << 31);
}

int32_t csd_attn_mfma_enqueue(csd_model *mod, const KvGeom &geo, const void *kv, const int32_t *cache_len, int B, int m,
                              int layer, float scale, const AttnMode &mode, hipStream_t st, bf16_t *out,
                              size_t out_plane);   // csd_attention.hip

int32_t csd_chain_enqueue(csd_model *mod, void *kv, const int32_t *tokens, const int32_t *cache_len, int32_t B, int32_t m,
                          float *logits, hipStream_t st) {
    const csd_model_cfg &c = mod->cfg;
    const int M = B * m, d = c.d_model, F = c.d_ffn, hd = mod->hd, V = c.vocab, L = c.n_layers;
    const bool t5 = c.arch == 1;     // T5-style decoder: no rotary embedding, biased unscaled scores, a cross-attention sub-layer
    const KvGeom geo{c.max_batch, c.n_heads, c.head_dim, mod->seq_pad, L, mod->kperm ? 1 : 0};
    const int mtp = mod->act_mtp;
    const int pb_d = (int)(mod->x_plane[0] * 2), pb_hd = (int)(mod->x_plane[1] * 2), pb_F = (int)(mod->x_plane[3] * 2);
    bf16_t *X1 = (bf16_t *)mod->x[0], *X2 = (bf16_t *)mod->x[1], *X3 = (bf16_t *)mod->x[2], *X4 = (bf16_t *)mod->x[3];
    float *ssq1 = mod->ssq[0], *ssq3 = mod->ssq[1];
    const float scale = t5 ? 1.0f : 1.0f / sqrtf((float)c.head_dim);
    const int ssq_rows = (M + 15) / 16 * 16;
    {
        ProfScope ps(mod, st, CSD_PROF_OTHER);
        hipLaunchKernelGGL(kc_embed, dim3(M), dim3(256), 0, st, tokens, (const bf16_t *)mod->embed, V, d, mod->layers[0].attn_norm,
                           mod->h, X1, pb_d, mtp, ssq1, ssq_rows, cache_len, m, c.head_dim, t5 ? 0.f : c.rope_theta, mod->rope,
                           mod->tree_call ? mod->tree_depth : nullptr);
        CSD_LAUNCH_CHECK();
    }
    if (mod->trace) CSD_HIP(hipMemcpyAsync(mod->trace, mod->h, sizeof(float) * (size_t)M * d, hipMemcpyDeviceToDevice, st));
    ChainGemm base{};
    base.mtp = mtp;
    base.M = M;
    base.inv_d = 1.0f / (float)d;
    base.eps = c.rms_eps;
    base.h = mod->h;
    base.d = d;
    base.m = m;
    base.hd = hd;
    base.dh = c.head_dim;
    base.geo = geo;
    base.cache_len = cache_len;
    base.rope = (!t5 && c.rope_theta > 0.f) ? mod->rope : nullptr;
    base.q = (bf16_t *)mod->qbuf;
    base.q_plane_bytes = (int)(mod->q_plane * 2);
    base.kv = (bf16_t *)kv;
    base.n_ssq = d / 16;
    base.ssq_rows = ssq_rows;
    auto gemm = [&](const GemmW &w, const bf16_t *a, int a_plane_bytes, const float *ssq_in) {
        ChainGemm P = base;
        P.Wp = (const u32x4 *)w.data;
        P.KS = w.K / 32;
        P.wbytes = (int)((size_t)w.K * w.N * 2);
        P.a = a;
        P.a_plane_bytes = a_plane_bytes;
        P.ssq_in = ssq_in;
        return P;
    };
    const AttnArgs attn{(const bf16_t *)mod->qbuf, (int)mod->q_plane, m, cache_len, geo, 0, (const bf16_t *)kv, scale, mod->attn_part,
                        mod->attn_chunks_max, mod->attn_cnt, mod->tree_call ? mod->tree_anc : nullptr, nullptr, 0, X2, pb_hd, mtp};
    int32_t rc;
    for (int l = 0; l < L; l++) {
        const LayerW &lw = mod->layers[l];
        ChainGemm Pq = gemm(lw.qkv, X1, pb_d, ssq1);
        Pq.layer = l;
        ChainGemm Po = gemm(lw.o, X2, pb_hd, nullptr);
        Po.gain = lw.ffn_norm;
        Po.out = X3;
        Po.out_plane_bytes = pb_d;
        Po.ssq_out = ssq3;
        ChainGemm Pg = gemm(lw.gu, X3, pb_d, ssq3);
        Pg.out = X4;
        Pg.out_plane_bytes = pb_F;
        ChainGemm Pd = gemm(lw.down, X4, pb_F, nullptr);
        Pd.gain = (l + 1 < L) ? mod->layers[l + 1].attn_norm : mod->final_norm;
        Pd.out = X1;
        Pd.out_plane_bytes = pb_d;
        Pd.ssq_out = ssq1;
        if (t5) {
            // QKV -> self-attention (bias by relative position) -> O (+h) -> cross-q -> cross-attention over the projected
            // encoder rows -> cross-O (+h) -> gate|up (tanh-GELU) -> down (+h): eight launches and two attention pairs
            AttnMode self_mode, cross_mode;
            self_mode.rel_bias = mod->rel_bias;
            self_mode.bucket = mod->rel_bucket;
            self_mode.bias_hd = mod->rel_bias_hd;
            cross_mode.fixed_nk = c.enc_len;
            const KvGeom cgeo{c.max_batch, c.n_heads, c.head_dim, mod->enc_pad, L, 0};
            const void *kv_cross = (const char *)kv + csd_self_kv_bytes(mod);
            Po.gain = lw.cross_norm;                           // the O projection feeds the cross-attention's norm
            ChainGemm Pcq = gemm(lw.cq, X3, pb_d, ssq3);       // queries only: the epilogue of QKV with one region
            Pcq.layer = l;
            ChainGemm Pco = gemm(lw.co, X2, pb_hd, nullptr);
            Pco.gain = lw.ffn_norm;
            Pco.out = X3;
            Pco.out_plane_bytes = pb_d;
            Pco.ssq_out = ssq3;
            Pg.gelu = 1;
#define CH_STEP(EPI_, P_, W_)                                                                   \
    {                                                                                           \
        ProfScope ps(mod, st, CSD_PROF_GEMM);                                                   \
        if ((rc = chain_launch<EPI_>(P_, (W_).N / 16, st)) != CSD_OK) return rc;               \
        CSD_LAUNCH_CHECK();                                                                     \
    }
            // either attention: the kernel whose last chunk merges, or (more than 16 rows per sequence, or so many chunks
            // that bandwidth rather than latency binds) the one with longer key runs and a merge kernel
            auto attention = [&](const KvGeom &g_, const void *kv_, int keys_pad, const AttnMode &mode) -> int32_t {
                const int chunks = (keys_pad + CA_KEYS - 1) / CA_KEYS;
                if ((long long)chunks * c.n_heads * B > 1024 || m > 16 || chunks > CA_MAX_CHUNKS)
                    return csd_attn_mfma_enqueue(mod, g_, kv_, cache_len, B, m, l, scale, mode, st, X2, mod->x_plane[1]);
                ProfScope ps(mod, st, CSD_PROF_ATTN);
                AttnArgs A = attn;
                A.geo = g_;
                A.kv = (const bf16_t *)kv_;
                A.layer = l;
                A.bias_hd = mode.bias_hd;
                A.fixed_nk = mode.fixed_nk;
                const dim3 grid(c.n_heads, B, chunks);     // chunk index slowest: see kc_attn
                if (c.head_dim == 128)
                    hipLaunchKernelGGL((kc_attn<128>), grid, dim3(256), 0, st, A);
                else
                    hipLaunchKernelGGL((kc_attn<64>), grid, dim3(256), 0, st, A);
                CSD_LAUNCH_CHECK();
                return CSD_OK;
            };
            CH_STEP(EPI_QKV, Pq, lw.qkv)
            if ((rc = attention(geo, kv, mod->seq_pad, self_mode)) != CSD_OK) return rc;
            CH_STEP(EPI_RESID, Po, lw.o)
            CH_STEP(EPI_QKV, Pcq, lw.cq)
            if ((rc = attention(cgeo, kv_cross, mod->enc_pad, cross_mode)) != CSD_OK) return rc;
            CH_STEP(EPI_RESID, Pco, lw.co)
            CH_STEP(EPI_GU, Pg, lw.gu)
            CH_STEP(EPI_RESID, Pd, lw.down)
#undef CH_STEP
            if (mod->trace)
                CSD_HIP(hipMemcpyAsync(mod->trace + (size_t)(l + 1) * M * d, mod->h, sizeof(float) * (size_t)M * d,
                                       hipMemcpyDeviceToDevice, st));
            continue;
        }
        AttnArgs A = attn;
        A.layer = l;
        const int chunks = (mod->seq_pad + CA_KEYS - 1) / CA_KEYS;           // chunk slots; those past a sequence's rows leave at once
        {
            {
                ProfScope ps(mod, st, CSD_PROF_GEMM);
                if ((rc = chain_launch<EPI_QKV>(Pq, lw.qkv.N / 16, st)) != CSD_OK) return rc;
                CSD_LAUNCH_CHECK();
            }
            if ((long long)chunks * c.n_heads * B > 1024 || m > 16) {
                // many sequences or long caches: the attention is bound by bandwidth, not by latency, and the kernel
                // with longer key runs per wave (and a merge kernel) moves the cache faster; it also takes the blocks of
                // more than 16 rows per sequence
                AttnMode am;
                if (mod->tree_call) am.anc = mod->tree_anc;
                if ((rc = csd_attn_mfma_enqueue(mod, geo, kv, cache_len, B, m, l, scale, am, st, X2, mod->x_plane[1])) != CSD_OK)
                    return rc;
            } else {
                ProfScope ps(mod, st, CSD_PROF_ATTN);
                const dim3 grid(c.n_heads, B, chunks);     // chunk index slowest: see kc_attn
                if (c.head_dim == 128)
                    hipLaunchKernelGGL((kc_attn<128>), grid, dim3(256), 0, st, A);
                else
                    hipLaunchKernelGGL((kc_attn<64>), grid, dim3(256), 0, st, A);
                CSD_LAUNCH_CHECK();
            }
            {
                ProfScope ps(mod, st, CSD_PROF_GEMM);
                if ((rc = chain_launch<EPI_RESID>(Po, lw.o.N / 16, st)) != CSD_OK) return rc;
                CSD_LAUNCH_CHECK();
            }
            {
                ProfScope ps(mod, st, CSD_PROF_GEMM);
                if ((rc = chain_launch<EPI_GU>(Pg, lw.gu.N / 16, st)) != CSD_OK) return rc;
                CSD_LAUNCH_CHECK();
            }
            {
                ProfScope ps(mod, st, CSD_PROF_GEMM);
                if ((rc = chain_launch<EPI_RESID>(Pd, lw.down.N / 16, st)) != CSD_OK) return rc;
                CSD_LAUNCH_CHECK();
            }
        }
        if (mod->trace)
            CSD_HIP(hipMemcpyAsync(mod->trace + (size_t)(l + 1) * M * d, mod->h, sizeof(float) * (size_t)M * d,
                                   hipMemcpyDeviceToDevice, st));
    }
    {
        ProfScope ps(mod, st, CSD_PROF_GEMM);
        ChainGemm P = gemm(mod->lm, X1, pb_d, ssq1);
        P.logits = logits;
        P.V = V;
        if ((rc = chain_launch<EPI_LOGITS>(P, mod->lm.N / 16, st)) != CSD_OK) return rc;
        CSD_LAUNCH_CHECK();
    }
    (void)F;
    return CSD_OK;
}
