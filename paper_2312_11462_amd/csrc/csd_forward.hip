// Review forward of the reviewing model over a drafted block (Section 2: one run scores all
// drafted positions), LLaMA-style decoder as the benchmark configurations describe it.
//
// Data flow per layer (M = B*m block rows, everything stays on the device):
//   a = rmsnorm(h) -> [QKV GEMM] -> rotate q,k; append K,V to the cache -> block attention
//   -> [O GEMM] -> h += ; a = rmsnorm(h) -> [gate/up GEMM] -> f = silu(g)*u -> [down GEMM] -> h +=
// The GEMMs stream each weight matrix from HBM exactly once.  With M <= 136 rows they are
// bandwidth-bound, so the work is split over (output-tile group, K slice) per wavefront, each
// wave streaming its own contiguous run of pre-tiled 1 KB weight fragments straight into MFMA
// operands; K slices write partial-sum planes that the small epilogue kernels add up in a fixed
// order (deterministic, no float atomics) while applying residual / norm / rotation / SwiGLU.
#include <cmath>

#include "csd_internal.h"

// ------------------------------------------------------------------------------ weight tiling

// One 16-byte chunk per thread: tile (nt, ks), lane (i = lane%16 -> output feature, g = lane/16)
// holds W[ks*32 + 8g + j][nt*16 + i], j = 0..7, the A operand of v_mfma_f32_16x16x32_bf16.
// perm_dh > 0: the piece is a q or k projection whose output features are taken in rotary pair order.
__global__ void k_pack_tiles(const bf16_t *__restrict__ src, int K, int N_src, bf16_t *__restrict__ dst, int KS,
                             int dst_tile_base, int dst_tile_stride, int perm_dh) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t total = (size_t)(N_src / 16) * KS * 64;
    if (idx >= total) return;
    const int lane = (int)(idx & 63);
    const int ks = (int)((idx >> 6) % KS);
    const int nt = (int)((idx >> 6) / KS);
    const int i = lane & 15, g = lane >> 4;
    const int dt = dst_tile_base + dst_tile_stride * nt;
    bf16_t *o = dst + (((size_t)dt * KS + ks) * 64 + lane) * 8;
    int col = nt * 16 + i;
    if (perm_dh > 0) {
        const int head = (nt * 16) / perm_dh, ti = nt % (perm_dh / 16);
        col = head * perm_dh + (i < 8 ? 8 * ti + i : perm_dh / 2 + 8 * ti + (i - 8));
    }
    const bf16_t *s = src + (size_t)(ks * 32 + 8 * g) * N_src + col;
#pragma unroll
    for (int j = 0; j < 8; j++) o[j] = s[(size_t)j * N_src];
}

template <typename T>
__global__ void k_copy_cols(const T *__restrict__ src, int K, int N_src, T *__restrict__ dst, int N_dst, int col0) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)K * N_src) return;
    const size_t k = idx / N_src, n = idx % N_src;
    dst[k * N_dst + col0 + n] = src[idx];
}

// ------------------------------------------------------------------------------------ GEMMs

// Weight-streaming GEMMs on the matrix cores.
//   A operand = weight fragment (16 output features x 32 k), B operand = activations
//   (32 k x 16 block rows), D = 16 features x 16 rows: lane (row = lane%16, features 4g..4g+3).
// Every form writes fp32 partial sums per K split ([S][M][N]); the epilogue kernels reduce them in a
// fixed order.

// Blocks of up to 32 rows (MT row tiles; the launcher instantiates NT = 1, MT = 1 and 2).  A workgroup covers 4 * NT adjacent output tiles of one K slice
// and shares the activation fragments through LDS: two chunks of U k-steps, laid out
// [chunk][u][row tile][hi|lo plane][lane] in MFMA operand order, so a fragment is one conflict-free 16-byte
// LDS read.  (A form with one independent wave per output tile re-read the activations from L2 in every
// wave and was slower from 6 rows on.)  The two jobs are given to different waves: waves 0-3 only stream
// weights (a register ring refilled k-step by k-step) and feed the matrix cores for all row tiles; waves
// 4-7 only move activation fragments from L2 to LDS, two chunks ahead in registers and one chunk ahead in
// LDS.  A wave that waits for its oldest load waits for nothing younger, so with the jobs apart the weight
// ring and the activation staging each keep their own depth.  One workgroup barrier per chunk hands a
// staged chunk over and frees the other buffer; both kinds of waves pass exactly 1 + (number of chunks)
// barriers.
template <int NT, int MT, int U>
__global__ __launch_bounds__(512) void k_gemm_ws(const u32x4 *__restrict__ Wp, const bf16_t *__restrict__ act, size_t plane,
                                                 int mtp, float *__restrict__ part, int M, int Mtot, int K, int N, int S) {
    extern __shared__ __align__(16) char wg_smem[];
    constexpr int CH = U * MT * 2 * 64;                      // 16-byte fragments per chunk
    static_assert(CH % 256 == 0, "chunk must divide over the staging waves");
    constexpr int ST = CH / 256;                             // staging loads per staging thread and chunk
    constexpr int PD = 4;                                    // LDS fragments are read this many (u, row tile) steps ahead
    static_assert(U * MT >= PD, "chunk shorter than the LDS prefetch distance");
    u32x4 *lbuf = reinterpret_cast<u32x4 *>(wg_smem);        // [2][CH]
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int s = blockIdx.x % S, grp = blockIdx.x / S;
    const int KS = K / 32, n_tiles = N / 16;
    const int ks0 = (int)((long long)KS * s / S), ks1 = (int)((long long)KS * (s + 1) / S);
    const int n_chunks = (ks1 - ks0 + U - 1) / U;
    const int t = lane & 15, g = lane >> 4;
    const u32x4 zero = u32x4{0u, 0u, 0u, 0u};

    if (w < 4) {
        // ------------------------------------------------------------ weight stream + matrix cores
        const int tile0 = (grp * 4 + w) * NT;
        // Every load below is issued unconditionally (the compiler can then count the loads in flight and wait
        // for exactly the oldest ones); what must not be read gets an offset beyond the buffer instead, which
        // touches no memory and returns zeros.
        const __amdgpu_buffer_rsrc_t rw =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<u32x4 *>(Wp), 0, (int)((size_t)K * N * sizeof(bf16_t)), 0x00020000);
        bool tv[NT];
        int wvoff[NT];
#pragma unroll
        for (int j = 0; j < NT; j++) {
            tv[j] = tile0 + j < n_tiles;
            wvoff[j] = tv[j] ? lane * 16 : (int)0x80000000;
        }
        f32x4 acc[MT][NT];
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
#pragma unroll
            for (int j = 0; j < NT; j++) acc[mt][j] = f32x4{0.f, 0.f, 0.f, 0.f};
        u32x4 wa[U][NT], wb[U][NT];

#define CSD_WS_LOAD_W1(WF, UU, KSU)                                                               \
    {                                                                                             \
        const int ksu_ = (KSU);                                                                   \
        const bool in_ = ksu_ < ks1; /* uniform */                                                \
        _Pragma("unroll") for (int j = 0; j < NT; j++)                                            \
            WF[UU][j] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(          \
                rw, in_ ? wvoff[j] : (int)0x80000000, in_ && tv[j] ? ((tile0 + j) * KS + ksu_) * 1024 : 0, 2)); \
    }
#define CSD_WS_LOAD_W(WF, KS_AT)                                                                  \
    _Pragma("unroll") for (int u = 0; u < U; u++) CSD_WS_LOAD_W1(WF, u, (KS_AT) + u)
#define CSD_WS_MMA(WF, BUF, KS_NEXT)                                                              \
    {                                                                                             \
        const u32x4 *lb_ = lbuf + (BUF) * CH + lane;                                              \
        u32x4 b_[PD + 1][2];                                                                      \
        _Pragma("unroll") for (int p = 0; p < PD; p++) {                                          \
            b_[p][0] = lb_[p * 128];                                                              \
            b_[p][1] = lb_[p * 128 + 64];                                                         \
        }                                                                                         \
        _Pragma("unroll") for (int idx = 0; idx < U * MT; idx++) {                                \
            if (idx + PD < U * MT) {                                                              \
                b_[(idx + PD) % (PD + 1)][0] = lb_[(idx + PD) * 128];                             \
                b_[(idx + PD) % (PD + 1)][1] = lb_[(idx + PD) * 128 + 64];                        \
            }                                                                                     \
            const int u = idx / MT, mt = idx % MT;                                                \
            _Pragma("unroll") for (int j = 0; j < NT; j++)                                        \
                acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(                             \
                    __builtin_bit_cast(bf16x8, WF[u][j]), __builtin_bit_cast(bf16x8, b_[idx % (PD + 1)][0]), acc[mt][j], 0, 0, 0); \
            _Pragma("unroll") for (int j = 0; j < NT; j++)                                        \
                acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(                             \
                    __builtin_bit_cast(bf16x8, WF[u][j]), __builtin_bit_cast(bf16x8, b_[idx % (PD + 1)][1]), acc[mt][j], 0, 0, 0); \
            if (mt == MT - 1) /* this k-step's weight registers are free: fetch the k-step 2 * U ahead */ \
                CSD_WS_LOAD_W1(WF, u, (KS_NEXT) + u)                                              \
            __builtin_amdgcn_sched_barrier(0);                                                    \
        }                                                                                         \
    }

        // the weight ring holds 2 * U k-steps and is refilled k-step by k-step, so every load is issued
        // 2 * U k-steps before its use
        CSD_WS_LOAD_W(wa, ks0)
        CSD_WS_LOAD_W(wb, ks0 + U)
        lds_sync();                                          // chunk 0 is in LDS
        for (int c = 0; c < n_chunks; c += 2) {
            CSD_WS_MMA(wa, 0, ks0 + (c + 2) * U)
            lds_sync();                                      // chunk c consumed, chunk c + 1 staged
            if (c + 1 >= n_chunks) break;
            CSD_WS_MMA(wb, 1, ks0 + (c + 3) * U)
            lds_sync();
        }
#undef CSD_WS_LOAD_W1
#undef CSD_WS_LOAD_W
#undef CSD_WS_MMA
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            const int row = mt * 16 + t;
            if (row < M) {
#pragma unroll
                for (int j = 0; j < NT; j++)
                    if (tv[j]) {
                        float *o = part + ((size_t)s * Mtot + row) * N + (size_t)(tile0 + j) * 16 + 4 * g;
                        *reinterpret_cast<f32x4 *>(o) = acc[mt][j];
                    }
            }
        }
    } else {
        // ------------------------------------------------------------ activation staging
        // fragment i * 256 + (tid - 256) of a chunk = (u, row tile, plane, lane) in that order: u, row tile
        // and plane are the same for a whole wave, so they go into the scalar offset of a buffer load (the
        // activations are stored fragment by fragment, see act_tiled_idx) and the per-lane part is one
        // register for all fragments.  Lanes of rows past M get an offset beyond the buffer: such loads
        // touch no memory and return zeros.
        const int sw = w - 4, stid = tid - 256;
        const __amdgpu_buffer_rsrc_t ra =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(act), 0, (int)(2 * plane * sizeof(bf16_t)), 0x00020000);
        const int voff_in = (4 * t + g) * 16;
        const int voff_last = ((MT - 1) * 16 + t < M) ? voff_in : (int)0x80000000;   // the last row tile may be ragged
        const int plane_off = (sw & 1) * (int)(plane * sizeof(bf16_t));
        u32x4 sa[ST], sb[ST];
#define CSD_WS_LOAD_ACT(SF, KS_AT)                                                                \
    _Pragma("unroll") for (int i = 0; i < ST; i++) {                                              \
        const int r2_ = i * 2 + (sw >> 1), mt_ = r2_ % MT, ksu_ = (KS_AT) + r2_ / MT;             \
        const int soff_ = plane_off + (ksu_ * mtp + mt_) * 1024;                                  \
        const bool in_ = ksu_ < ks1; /* uniform; past the slice: an offset beyond the buffer */   \
        SF[i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(                  \
            ra, !in_ ? (int)0x80000000 : mt_ == MT - 1 ? voff_last : voff_in, in_ ? soff_ : 0, 0)); \
    }
#define CSD_WS_PUT_ACT(SF, BUF)                                                                   \
    _Pragma("unroll") for (int i = 0; i < ST; i++) lbuf[(BUF) * CH + i * 256 + stid] = SF[i];

        CSD_WS_LOAD_ACT(sa, ks0)
        CSD_WS_LOAD_ACT(sb, ks0 + U)
        CSD_WS_PUT_ACT(sa, 0)
        lds_sync();
        for (int c = 0; c < n_chunks; c += 2) {
            CSD_WS_LOAD_ACT(sa, ks0 + (c + 2) * U)
            CSD_WS_PUT_ACT(sb, 1)                            // chunk c + 1, fetched one round ago
            lds_sync();
            if (c + 1 >= n_chunks) break;
            CSD_WS_LOAD_ACT(sb, ks0 + (c + 3) * U)
            CSD_WS_PUT_ACT(sa, 0)
            lds_sync();
        }
#undef CSD_WS_LOAD_ACT
#undef CSD_WS_PUT_ACT
    }
}

// Blocks of 33 to 144 rows (3 to 9 row tiles), where the matrix cores and LDS bandwidth matter as much as HBM: the
// rows are split over the 4 compute waves (RW row tiles each) and the weights are what is shared.  Waves
// 4-7 stream the weight fragments of CT column tiles from HBM into LDS (two chunks ahead in registers, one
// in LDS); a compute wave keeps its own rows' activation fragments in registers (fetched from L2 one chunk
// of k-steps ahead, slot by slot as they are used up) and reads every weight fragment once from LDS for
// 2 * RW matrix instructions: with two row tiles per wave the matrix cores get four instructions per
// 16-byte LDS read, where the activation-sharing form above gets two (its LDS reads then take as long as
// its matrix instructions), and nothing goes through LDS that only one wave needs.
template <int CT, int RW, int U>
__global__ __launch_bounds__(512) void k_gemm_rs(const u32x4 *__restrict__ Wp, const bf16_t *__restrict__ act, size_t plane,
                                                 int mtp, float *__restrict__ part, int M, int Mtot, int K, int N, int S) {
    extern __shared__ __align__(16) char wg_smem[];
    constexpr int CH = U * CT * 64;                          // 16-byte weight fragments (per lane) of a chunk
    constexpr int ST = CH / 256;                             // staging loads per staging thread and chunk
    constexpr int PD = 3;                                    // LDS reads run this many column tiles ahead
    static_assert(CH % 256 == 0 && U * CT > PD, "chunk shape");
    u32x4 *lbuf = reinterpret_cast<u32x4 *>(wg_smem);        // [2][CH]
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int s = blockIdx.x % S, grp = blockIdx.x / S;
    const int KS = K / 32, n_tiles = N / 16;
    const int ks0 = (int)((long long)KS * s / S), ks1 = (int)((long long)KS * (s + 1) / S);
    const int n_chunks = (ks1 - ks0 + U - 1) / U;
    const int t = lane & 15, g = lane >> 4;
    const int tile0 = grp * CT;
    const u32x4 zero = u32x4{0u, 0u, 0u, 0u};

    if (w < 4) {
        // ------------------------------------------------------------ own rows x all column tiles
        const __amdgpu_buffer_rsrc_t ra =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(act), 0, (int)(2 * plane * sizeof(bf16_t)), 0x00020000);
        const int lo_off = (int)(plane * sizeof(bf16_t));
        int voff[RW];                                        // rows past M: an offset beyond the buffer (loads give 0)
#pragma unroll
        for (int r = 0; r < RW; r++) {
            const int row = (w * RW + r) * 16 + t;
            voff[r] = row < M ? (4 * t + g) * 16 : (int)0x80000000;
        }
        const bool has_rows = w * RW * 16 < M;               // uniform
        f32x4 acc[RW][CT];
#pragma unroll
        for (int r = 0; r < RW; r++)
#pragma unroll
            for (int ct = 0; ct < CT; ct++) acc[r][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
        u32x4 a[U][RW][2];

#define CSD_RS_LOAD_A(UU, KS_AT)                                                                  \
    {                                                                                             \
        const int ksa_ = (KS_AT);                                                                 \
        const bool in_ = ksa_ < ks1; /* uniform; past the slice: an offset beyond the buffer, no branch */ \
        _Pragma("unroll") for (int r = 0; r < RW; r++) {                                          \
            const int vo_ = in_ ? voff[r] : (int)0x80000000;                                      \
            const int so_ = in_ ? (ksa_ * mtp + w * RW + r) * 1024 : 0; /* one stored fragment, see act_tiled_idx */ \
            a[UU][r][0] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(ra, vo_, so_, 0)); \
            a[UU][r][1] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(ra, vo_, in_ ? so_ + lo_off : 0, 0)); \
        }                                                                                         \
    }
#define CSD_RS_MMA(BUF, KS_NEXT)                                                                  \
    if (has_rows) {                                                                               \
        const u32x4 *lb_ = lbuf + (BUF) * CH + lane;                                              \
        u32x4 wf_[PD + 1];                                                                        \
        _Pragma("unroll") for (int p = 0; p < PD; p++) wf_[p] = lb_[p * 64];                      \
        _Pragma("unroll") for (int idx = 0; idx < U * CT; idx++) {                                \
            if (idx + PD < U * CT) wf_[(idx + PD) % (PD + 1)] = lb_[(idx + PD) * 64];             \
            const int u = idx / CT, ct = idx % CT;                                                \
            _Pragma("unroll") for (int r = 0; r < RW; r++)                                        \
                acc[r][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(                             \
                    __builtin_bit_cast(bf16x8, wf_[idx % (PD + 1)]), __builtin_bit_cast(bf16x8, a[u][r][0]), acc[r][ct], 0, 0, 0); \
            _Pragma("unroll") for (int r = 0; r < RW; r++)                                        \
                acc[r][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(                             \
                    __builtin_bit_cast(bf16x8, wf_[idx % (PD + 1)]), __builtin_bit_cast(bf16x8, a[u][r][1]), acc[r][ct], 0, 0, 0); \
            if (ct == CT - 1) CSD_RS_LOAD_A(u, (KS_NEXT) + u) /* slot u is free: k-step U ahead */  \
            if (RW != 3 || (idx & 3) == 3) __builtin_amdgcn_sched_barrier(0);                    \
        }                                                                                         \
    }

        if (has_rows) {
#pragma unroll
            for (int u = 0; u < U; u++) CSD_RS_LOAD_A(u, ks0 + u)
        }
        lds_sync();                                          // weight chunk 0 is in LDS
        for (int c = 0; c < n_chunks; c += 2) {
            CSD_RS_MMA(0, ks0 + (c + 1) * U)
            lds_sync();                                      // chunk c consumed, chunk c + 1 staged
            if (c + 1 >= n_chunks) break;
            CSD_RS_MMA(1, ks0 + (c + 2) * U)
            lds_sync();
        }
#undef CSD_RS_LOAD_A
#undef CSD_RS_MMA
#pragma unroll
        for (int r = 0; r < RW; r++) {
            const int row = (w * RW + r) * 16 + t;
            if (row < M) {
#pragma unroll
                for (int ct = 0; ct < CT; ct++)
                    if (tile0 + ct < n_tiles) {
                        float *o = part + ((size_t)s * Mtot + row) * N + (size_t)(tile0 + ct) * 16 + 4 * g;
                        *reinterpret_cast<f32x4 *>(o) = acc[r][ct];
                    }
            }
        }
    } else {
        // ------------------------------------------------------------ weight staging
        // fragment i * 256 + (tid - 256) of a chunk = (u, column tile, lane): u and the tile are the same
        // for a whole wave and go into the scalar offset
        const int sw = w - 4, stid = tid - 256;
        const __amdgpu_buffer_rsrc_t rw =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<u32x4 *>(Wp), 0, (int)((size_t)K * N * sizeof(bf16_t)), 0x00020000);
        const int voff = lane * 16;
        u32x4 sa[ST], sb[ST];
#define CSD_RS_LOAD_W(SF, KS_AT)                                                                  \
    _Pragma("unroll") for (int i = 0; i < ST; i++) {                                              \
        const int rest_ = i * 4 + sw, tile_ = tile0 + rest_ % CT, ksu_ = (KS_AT) + rest_ / CT;    \
        const bool in_ = ksu_ < ks1 && tile_ < n_tiles; /* uniform; else an offset beyond the buffer */ \
        SF[i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(                  \
            rw, in_ ? voff : (int)0x80000000, in_ ? (tile_ * KS + ksu_) * 1024 : 0, 2));          \
    }
#define CSD_RS_PUT_W(SF, BUF)                                                                     \
    _Pragma("unroll") for (int i = 0; i < ST; i++) lbuf[(BUF) * CH + i * 256 + stid] = SF[i];

        CSD_RS_LOAD_W(sa, ks0)
        CSD_RS_LOAD_W(sb, ks0 + U)
        CSD_RS_PUT_W(sa, 0)
        lds_sync();
        for (int c = 0; c < n_chunks; c += 2) {
            CSD_RS_LOAD_W(sa, ks0 + (c + 2) * U)
            CSD_RS_PUT_W(sb, 1)                              // chunk c + 1, fetched one round ago
            lds_sync();
            if (c + 1 >= n_chunks) break;
            CSD_RS_LOAD_W(sb, ks0 + (c + 3) * U)
            CSD_RS_PUT_W(sa, 0)
            lds_sync();
        }
#undef CSD_RS_LOAD_W
#undef CSD_RS_PUT_W
    }
}

// Generic GEMM (fp32 models and the debugging path): one thread per output column, fp32
// activations [M][K], row-major weights [K][N]; writes partial plane 0.
template <typename TW>
__global__ __launch_bounds__(256) void k_gemm_simple(const TW *__restrict__ W, const float *__restrict__ act,
                                                     float *__restrict__ part, int M, int K, int N) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    for (int r0 = 0; r0 < M; r0 += 8) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        const int rn = min(8, M - r0);
        for (int k = 0; k < K; k++) {
            const float w = to_f32<TW>(W[(size_t)k * N + n]);
#pragma unroll
            for (int r = 0; r < 8; r++)
                if (r < rn) acc[r] = fmaf(act[(size_t)(r0 + r) * K + k], w, acc[r]);
        }
        for (int r = 0; r < rn; r++) part[(size_t)(r0 + r) * N + n] = acc[r];
    }
}

// ------------------------------------------------------------------------------- epilogues

// h[r] = E[token[r]];  a[r] = h[r] * g and rstd[r] = 1 / sqrt(mean(h[r]^2) + eps): the norm is folded around the
// GEMM that follows, rmsnorm(h) * g @ W = rstd * ((h * g) @ W), so that what is rounded to the two bf16 planes is
// h * g (exact for embedding rows with unit gains) and the scale is applied to fp32 sums by the GEMM's epilogue kernel.
template <typename TW, typename TA>
__global__ __launch_bounds__(256) void k_embed_norm(const int32_t *__restrict__ tokens, const TW *__restrict__ E, int V,
                                                    int d, const float *__restrict__ g, float eps,
                                                    float *__restrict__ h, TA *__restrict__ a, int lda, size_t plane, int mtp,
                                                    float *__restrict__ rstd) {
    __shared__ float red[16];
    const int r = blockIdx.x;
    const int tok = tokens[r];
    const bool ok = tok >= 0 && tok < V;
    float ss = 0.f;
    for (int x = threadIdx.x; x < d; x += blockDim.x) {
        const float v = ok ? to_f32<TW>(E[(size_t)tok * d + x]) : 0.f;
        h[(size_t)r * d + x] = v;
        ss += v * v;
    }
    ss = block_sum(ss, red);
    if (threadIdx.x == 0) rstd[r] = rsqrtf(ss / (float)d + eps);
    for (int x = threadIdx.x; x < d; x += blockDim.x)
        store_act<TA>(a, plane, r, x, lda, mtp, h[(size_t)r * d + x] * g[x]);
}

// h[r] += sum_s part[s][r];  a[r] = h[r] * g, rstd[r] as above.  One workgroup of 1024 threads per row, four
// consecutive features per thread and pass (16-byte loads when d allows), the new h kept in registers
// between the sum of squares and the scaling for rows of up to RN_THREADS * 4 * RN_PASSES features.
#define RN_THREADS 1024
#define RN_PASSES 2
template <typename TA>
__global__ __launch_bounds__(RN_THREADS) void k_residual_norm(const float *__restrict__ part, int S, int M, int d,
                                                              const float *__restrict__ g, float eps, float *__restrict__ h,
                                                              TA *__restrict__ a, int lda, size_t plane, int mtp,
                                                              float *__restrict__ rstd) {
    __shared__ float red[RN_THREADS / 64];
    const int r = blockIdx.x;
    float ss = 0.f;
    if (d % 4 == 0 && d <= RN_THREADS * 4 * RN_PASSES) {
        f32x4 keep[RN_PASSES], gain[RN_PASSES];              // the gains are fetched with the sums, not after the reduction
#pragma unroll
        for (int p = 0; p < RN_PASSES; p++) {
            const int x = (p * RN_THREADS + (int)threadIdx.x) * 4;
            keep[p] = gain[p] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (x < d) {
                gain[p] = *reinterpret_cast<const f32x4 *>(g + x);
                f32x4 v = *reinterpret_cast<const f32x4 *>(h + (size_t)r * d + x);
                for (int s = 0; s < S; s++) v += *reinterpret_cast<const f32x4 *>(part + ((size_t)s * M + r) * d + x);
                *reinterpret_cast<f32x4 *>(h + (size_t)r * d + x) = v;
                keep[p] = v;
                ss += (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]);
            }
        }
        ss = block_sum(ss, red);
        if (threadIdx.x == 0) rstd[r] = rsqrtf(ss / (float)d + eps);
#pragma unroll
        for (int p = 0; p < RN_PASSES; p++) {
            const int x = (p * RN_THREADS + (int)threadIdx.x) * 4;
            if (x < d) {
                store_act4<TA>(a, plane, r, x, lda, mtp, keep[p] * gain[p]);
            }
        }
        return;
    }
    for (int x = threadIdx.x; x < d; x += blockDim.x) {
        float v = 0.f;
        for (int s = 0; s < S; s++) v += part[((size_t)s * M + r) * d + x];
        v += h[(size_t)r * d + x];
        h[(size_t)r * d + x] = v;
        ss += v * v;
    }
    ss = block_sum(ss, red);
    if (threadIdx.x == 0) rstd[r] = rsqrtf(ss / (float)d + eps);
    for (int x = threadIdx.x; x < d; x += blockDim.x)
        store_act<TA>(a, plane, r, x, lda, mtp, h[(size_t)r * d + x] * g[x]);
}

// bias_hd[h][n] = rel_bias[bucket[n]][h]: the relative-position bias of head h at look-back distance n
__global__ void k_bias_table(const float *__restrict__ rel_bias, const int32_t *__restrict__ bucket, int H,
                             float *__restrict__ bias_hd) {
    bias_hd[blockIdx.x * 128 + threadIdx.x] = rel_bias[bucket[threadIdx.x] * H + blockIdx.x];
}

// (cos, sin) of the rotary angle pos * theta^(-2x/dh) of every block row of a call and every pair x < dh/2,
// evaluated in double precision once per call instead of once per layer and head.
__global__ void k_rope_table(const int32_t *__restrict__ cache_len, int m, int dh, float theta, float2 *__restrict__ tab,
                             const int32_t *__restrict__ depth) {
    const int r = blockIdx.x, half = dh / 2;
    // the position of a row: where it sits in a plain block, how far it is from row 0 in a tree block
    const int pos = cache_len[r / m] + (depth ? depth[r] : r % m);
    for (int x = threadIdx.x; x < half; x += blockDim.x) {
        const double ang = (double)pos * pow((double)theta, -2.0 * (double)x / (double)dh);
        tab[(size_t)r * half + x] = float2{(float)cos(ang), (float)sin(ang)};
    }
}

// Sum the QKV partial planes, rotate q and k (half-split pairs, angles from k_rope_table; no table: no
// rotation), write q for the attention kernel and append K (rotated) and V to the cache at position
// cache_len[b] + i.
template <typename TA, typename TC>
__global__ __launch_bounds__(64) void k_fix_qkv(const float *__restrict__ part, int S, int M, int m,
                                                const int32_t *__restrict__ cache_len, KvGeom geo, int layer,
                                                const float2 *__restrict__ rope, TA *__restrict__ qout, size_t qplane,
                                                TC *__restrict__ kv, const float *__restrict__ rstd) {
    const int r = blockIdx.x, hh = blockIdx.y;
    const float rs = rstd[r];                            // the norm folded around the GEMM: scale its fp32 sums
    const int b = r / m, i = r % m;
    const int dh = geo.dh, half = dh / 2, hd = geo.H * dh, N = 3 * hd;
    const int pos = cache_len[b] + i;
    const bool pos_ok = pos >= 0 && pos < geo.seq_pad;
    TC *kc = kv + kv_k_off(geo, layer, b, hh);
    TC *vc = kv + kv_v_off(geo, layer, b, hh);
    for (int x = threadIdx.x; x < half; x += blockDim.x) {
        float q0 = 0.f, q1 = 0.f, k0 = 0.f, k1 = 0.f, v0 = 0.f, v1 = 0.f;
        const int p0 = rope_perm(x, dh, geo.kperm), p1 = rope_perm(x + half, dh, geo.kperm);
        for (int s = 0; s < S; s++) {
            const float *p = part + ((size_t)s * M + r) * N + hh * dh;
            q0 += p[p0];
            q1 += p[p1];
            k0 += p[hd + p0];
            k1 += p[hd + p1];
            v0 += p[2 * hd + x];
            v1 += p[2 * hd + x + half];
        }
        q0 *= rs, q1 *= rs, k0 *= rs, k1 *= rs, v0 *= rs, v1 *= rs;
        float c = 1.f, sn = 0.f;                         // no table: a model without rotary embedding
        if (rope) {
            const float2 cs = rope[(size_t)r * half + x];
            c = cs.x;
            sn = cs.y;
        }
        store_act<TA>(qout, qplane, r, hh * dh + p0, hd, 0, q0 * c - q1 * sn);
        store_act<TA>(qout, qplane, r, hh * dh + p1, hd, 0, q0 * sn + q1 * c);
        if (pos_ok) {
            kc[(size_t)pos * dh + p0] = from_f32<TC>(k0 * c - k1 * sn);
            kc[(size_t)pos * dh + p1] = from_f32<TC>(k0 * sn + k1 * c);
            vc[kv_v_idx(geo, x, pos)] = from_f32<TC>(v0);
            vc[kv_v_idx(geo, x + half, pos)] = from_f32<TC>(v1);
        }
    }
}

// f = silu(sum_s gate) * (sum_s up).  Tiled weights interleave gate and up tiles of 16 columns
// (gate tile j at packed tile 2j, up tile at 2j+1); row-major weights concatenate [gate | up].
template <typename TA>
__global__ __launch_bounds__(256) void k_fix_gu(const float *__restrict__ part, int S, int M, int F, int interleaved,
                                                TA *__restrict__ f, int ldf, size_t plane, int mtp, int gelu,
                                                const float *__restrict__ rstd) {
    const int r = blockIdx.y;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= F) return;
    const int gc = interleaved ? (j / 16) * 32 + (j % 16) : j;
    const int uc = interleaved ? gc + 16 : F + j;
    float gsum = 0.f, usum = 0.f;
    for (int s = 0; s < S; s++) {
        const float *p = part + ((size_t)s * M + r) * (2 * (size_t)F);
        gsum += p[gc];
        usum += p[uc];
    }
    gsum *= rstd[r], usum *= rstd[r];                    // the folded norm
    // gate activation: SiLU, or (arch 1) the tanh form of GELU
    const float sg = gelu ? 0.5f * gsum * (1.0f + tanhf(0.7978845608028654f * (gsum + 0.044715f * gsum * gsum * gsum)))
                          : gsum / (1.0f + expf(-gsum));
    store_act<TA>(f, plane, r, j, ldf, mtp, sg * usum);
}

__global__ __launch_bounds__(256) void k_fix_logits(const float *__restrict__ part, int S, int M, int V,
                                                    float *__restrict__ logits, const float *__restrict__ rstd) {
    const int r = blockIdx.y;
    const int v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= V) return;
    float acc = 0.f;
    for (int s = 0; s < S; s++) acc += part[((size_t)s * M + r) * V + v];
    logits[(size_t)r * V + v] = acc * rstd[r];           // the folded final norm
}

// out[r][j] = sum_s part[s][r][j] (two bf16 planes on the MFMA path): the cross-attention queries of arch 1
template <typename TA>
__global__ __launch_bounds__(256) void k_fix_plain(const float *__restrict__ part, int S, int M, int N, TA *__restrict__ out,
                                                   int ldo, size_t plane, const float *__restrict__ rstd) {
    const int r = blockIdx.y;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= N) return;
    float acc = 0.f;
    for (int s = 0; s < S; s++) acc += part[((size_t)s * M + r) * N + j];
    store_act<TA>(out, plane, r, j, ldo, 0, acc * rstd[r]);      // the folded norm
}

// arch 1, once per prompt: rows [row0, row0 + M) of the projected encoder output, part[s][r][0..hd) = keys and
// [hd..2hd) = values, go into the cross-attention part of the cache (keys row-major, values transposed)
template <typename TC>
__global__ __launch_bounds__(256) void k_fix_cross_kv(const float *__restrict__ part, int S, int M, KvGeom geo, int layer,
                                                      int b, int row0, TC *__restrict__ kvc) {
    const int r = blockIdx.y;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    const int hd = geo.H * geo.dh;
    if (j >= hd) return;
    float k = 0.f, v = 0.f;
    for (int s = 0; s < S; s++) {
        const float *p = part + ((size_t)s * M + r) * (2 * (size_t)hd);
        k += p[j];
        v += p[hd + j];
    }
    const int hh = j / geo.dh, x = j % geo.dh, pos = row0 + r;
    kvc[kv_k_off(geo, layer, b, hh) + (size_t)pos * geo.dh + x] = from_f32<TC>(k);
    kvc[kv_v_off(geo, layer, b, hh) + kv_v_idx(geo, x, pos)] = from_f32<TC>(v);
}

// a[r][x] = src[r][x] as GEMM input rows (two bf16 planes on the MFMA path)
template <typename TA>
__global__ __launch_bounds__(256) void k_rows_to_act(const float *__restrict__ src, int M, int d, TA *__restrict__ a, int lda,
                                                     size_t plane, int mtp) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)M * d) return;
    store_act<TA>(a, plane, (int)(idx / d), (int)(idx % d), lda, mtp, src[idx]);
}

// Generic causal block attention: one wave per (block row, head).  Scores of the visible cache
// rows 0..pos go through LDS; softmax in fp32 with max subtraction; o = sum_j p_j V_j.
template <typename TA, typename TC>
__global__ __launch_bounds__(64) void k_attn_simple(const TA *__restrict__ q, int m, const int32_t *__restrict__ cache_len,
                                                    KvGeom geo, int layer, const TC *__restrict__ kv, float scale,
                                                    size_t qplane, TA *__restrict__ out, int ldo, size_t plane, int mtp,
                                                    AttnMode mode) {
    extern __shared__ float sm[];
    const int r = blockIdx.x, hh = blockIdx.y;
    const int b = r / m, i = r % m;
    const int dh = geo.dh, hd = geo.H * dh;
    float *qs = sm;           // [dh]
    float *sc = sm + dh;      // [nk]
    const int qpos = mode.fixed_nk > 0 ? 0 : cache_len[b] + i;
    int nk = mode.fixed_nk > 0 ? mode.fixed_nk : qpos + 1;
    nk = max(1, min(nk, geo.seq_pad));
    const unsigned long long anc_row = mode.anc ? mode.anc[r] : 0ull;
    const int t0 = qpos - i;
    const TC *kc = kv + kv_k_off(geo, layer, b, hh);
    const TC *vc = kv + kv_v_off(geo, layer, b, hh);
    for (int x = threadIdx.x; x < dh; x += 64) {
        const size_t qi = (size_t)r * hd + hh * dh + x;
        qs[x] = to_f32<TA>(q[qi]) + (sizeof(TA) == 2 ? to_f32<TA>(q[qi + qplane]) : 0.f);
    }
    __syncthreads();
    float mx = -INFINITY;
    for (int j = threadIdx.x; j < nk; j += 64) {
        float s = 0.f;
        for (int x = 0; x < dh; x++) s = fmaf(qs[x], to_f32<TC>(kc[(size_t)j * dh + x]), s);
        s *= scale;
        if (mode.rel_bias) s += mode.rel_bias[mode.bucket[min(qpos - j, 127)] * geo.H + hh];
        if (mode.anc && !tree_sees(anc_row, j, t0)) s = -INFINITY;     // a row of the block that is not above this one
        sc[j] = s;
        mx = fmaxf(mx, s);
    }
    mx = wave_max(mx);
    float z = 0.f;
    for (int j = threadIdx.x; j < nk; j += 64) {
        const float e = expf(sc[j] - mx);
        sc[j] = e;
        z += e;
    }
    z = wave_sum(z);
    __syncthreads();
    const float rz = 1.0f / z;
    for (int x = threadIdx.x; x < dh; x += 64) {
        float o = 0.f;
        for (int j = 0; j < nk; j++) o = fmaf(sc[j], to_f32<TC>(vc[kv_v_idx(geo, x, j)]), o);
        store_act<TA>(out, plane, r, hh * dh + x, ldo, mtp, o * rz);
    }
}

// cache row import / export in canonical [n][H*dh] fp32 form
template <typename TC>
__global__ void k_kv_write(TC *__restrict__ kv, KvGeom geo, int layer, int b, int pos0, int n,
                           const float *__restrict__ K, const float *__restrict__ V) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int hd = geo.H * geo.dh;
    if (idx >= (size_t)n * hd) return;
    const int i = (int)(idx / hd), c = (int)(idx % hd), hh = c / geo.dh, x = c % geo.dh;
    kv[kv_k_off(geo, layer, b, hh) + (size_t)(pos0 + i) * geo.dh + rope_perm(x, geo.dh, geo.kperm)] = from_f32<TC>(K[idx]);
    kv[kv_v_off(geo, layer, b, hh) + kv_v_idx(geo, x, pos0 + i)] = from_f32<TC>(V[idx]);
}
template <typename TC>
__global__ void k_kv_read(const TC *__restrict__ kv, KvGeom geo, int layer, int b, int pos0, int n,
                          float *__restrict__ K, float *__restrict__ V) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int hd = geo.H * geo.dh;
    if (idx >= (size_t)n * hd) return;
    const int i = (int)(idx / hd), c = (int)(idx % hd), hh = c / geo.dh, x = c % geo.dh;
    K[idx] = to_f32<TC>(kv[kv_k_off(geo, layer, b, hh) + (size_t)(pos0 + i) * geo.dh + rope_perm(x, geo.dh, geo.kperm)]);
    V[idx] = to_f32<TC>(kv[kv_v_off(geo, layer, b, hh) + kv_v_idx(geo, x, pos0 + i)]);
}

// ------------------------------------------------------------------------------- host driver

static KvGeom geom(const csd_model *mod) {
    return KvGeom{mod->cfg.max_batch, mod->cfg.n_heads, mod->cfg.head_dim, mod->seq_pad, mod->cfg.n_layers,
                  mod->kperm ? 1 : 0};
}

ProfScope::ProfScope(csd_model *mod, hipStream_t s, int cls) : m(mod), st(s), on(false) {
    if (!mod->prof || mod->ev_used + 2 > mod->ev.size()) return;
    on = true;
    mod->ev_class.push_back(cls);
    (void)hipEventRecord(mod->ev[mod->ev_used], st);
}
ProfScope::~ProfScope() {
    if (!on) return;
    (void)hipEventRecord(m->ev[m->ev_used + 1], st);
    m->ev_used += 2;
}

#define WG_U_MAX 4      /* k-steps per chunk of the workgroup-tiled GEMMs */
template <int MT>
static int32_t launch_gemm_ws_mt(const GemmW &w, const bf16_t *act, size_t plane, int mtp, float *part, int M, int Mtot, int S,
                                 int groups, hipStream_t st) {
    const size_t lds = (size_t)2 * WG_U_MAX * MT * 2 * 64 * 16;      // allowed at csd_gemm_setup
    hipLaunchKernelGGL((k_gemm_ws<1, MT, WG_U_MAX>), dim3(groups * S), dim3(512), lds, st, reinterpret_cast<const u32x4 *>(w.data),
                       act, plane, mtp, part, M, Mtot, w.K, w.N, S);
    return CSD_OK;
}

// Blocks of up to 32 rows (of Mtot in the call): one column tile per wave, 64 columns per workgroup; K is split
// until there are two workgroups per compute unit: the light workgroups share a compute unit, and two per unit stream
// faster than one (measured: 3.84 -> 3.69 ms per step at 6 rows of the 7B shape; beyond 512 the partial sums cost
// more).  Two column tiles per wave, 128 columns per workgroup, were slower here (4.02 against 3.86 ms at 6 rows,
// 5.83 against 5.68 ms at 24 rows of batch 8).  *S_io: the number of K splits, chosen here when 0 (later row chunks
// of the same call must use the same).
static int32_t launch_gemm_ws(const GemmW &w, const bf16_t *act, size_t plane, int mtp, float *part, int M, int Mtot, int *S_io,
                              hipStream_t st) {
    const int n_tiles = w.N / 16, KS = w.K / 32, groups = (n_tiles + 3) / 4;
    int S = *S_io;
    if (S == 0) {
        S = 1;
        while (groups * S < 512 && S * 2 <= w.S && KS / (S * 2) >= 2 * WG_U_MAX) S *= 2;
        *S_io = S;
    }
    switch ((M + 15) / 16) {
    case 1: return launch_gemm_ws_mt<1>(w, act, plane, mtp, part, M, Mtot, S, groups, st);
    case 2: return launch_gemm_ws_mt<2>(w, act, plane, mtp, part, M, Mtot, S, groups, st);
    default: return CSD_ESHAPE;       // taller blocks take the row-split form
    }
}

template <int CT, int RW>
static int32_t launch_gemm_rs_t(const GemmW &w, const bf16_t *act, size_t plane, int mtp, float *part, int M, int Mtot, int S,
                                int groups, hipStream_t st) {
    const size_t lds = (size_t)2 * WG_U_MAX * CT * 64 * 16;          // allowed at csd_gemm_setup
    hipLaunchKernelGGL((k_gemm_rs<CT, RW, WG_U_MAX>), dim3(groups * S), dim3(512), lds, st, reinterpret_cast<const u32x4 *>(w.data),
                       act, plane, mtp, part, M, Mtot, w.K, w.N, S);
    return CSD_OK;
}

// The row-split form.  Its launches are bound by the matrix instructions of the busiest compute wave, so what
// matters is how many compute units have a workgroup: the column tiles per workgroup (CT) and the K splits (S, at most
// 8: the partial sums are traffic too) are chosen per matrix so that the launch comes as close to one workgroup per
// compute unit as the shape allows, the wider workgroup winning a tie (it reads the activation rows less often).
// Measured per launch at 128 rows of the 7B shape, against 16 tiles and 128 workgroups for every matrix: QKV 40.6 ->
// 33.1 us (12 tiles, 4 splits, 256 workgroups), O and down 30.6 -> 23.6 (8, 8, 256), gate|up 57.2 -> 49.1 (11, 2, 252).
static int rs_splits(int groups, int KS, int Mtot, int N, size_t part_floats) {
    int S = 1;
    while (groups * (S + 1) <= 256 && S < 8 && KS / (S + 1) >= 2 * WG_U_MAX && (size_t)(S + 1) * Mtot * N <= part_floats) S++;
    return S;
}
// rows: the rows of this launch (33 to 144), Mtot: the rows of the whole call (the partial-sum buffer holds S x Mtot x N
// floats), S_fixed: the number of splits when an earlier row chunk of the call has chosen it, else 0.
static void rs_plan(int N, int K, int rows, int Mtot, size_t part_floats, int S_fixed, int *ct_out, int *S_out) {
    const int n_tiles = N / 16, KS = K / 32, MT = (rows + 15) / 16;
    const int rw = MT <= 8 ? 2 : 3;          // row tiles per compute wave: waves past the block's rows only pass the barriers
    static const int cts2[] = {16, 12, 11, 8, 6, 0}, cts3[] = {8, 6, 0};
    const int *cts = rw == 2 ? cts2 : cts3;
    int ct = cts[0], S = S_fixed;
    double best = -1.0;
    for (int i = 0; cts[i]; i++) {
        const int groups = (n_tiles + cts[i] - 1) / cts[i];
        const int s = S_fixed ? S_fixed : rs_splits(groups, KS, Mtot, N, part_floats);
        const int wgs = groups * s;
        const double fill = (double)wgs / (256.0 * ((wgs + 255) / 256));
        if (fill > best) best = fill, ct = cts[i], S = s;
    }
    *ct_out = ct;
    *S_out = S;
}
int32_t csd_rs_plan_host(int32_t N, int32_t K, int32_t rows, size_t part_floats, int32_t *ct, int32_t *S) {
    if (!ct || !S) return CSD_ENULL;
    if (N <= 0 || K <= 0 || N % 16 || K % 32 || rows < 1 || rows > 144) return CSD_EINVAL;
    int c = 0, s = 0;
    rs_plan(N, K, rows, rows, part_floats, 0, &c, &s);
    *ct = c;
    *S = s;
    return CSD_OK;
}
static int32_t launch_gemm_rs(const csd_model *mod, const GemmW &w, const bf16_t *act, size_t plane, int mtp, float *part, int M,
                              int Mtot, int *S_io, hipStream_t st) {
    const int n_tiles = w.N / 16, MT = (M + 15) / 16;
    const int rw = MT <= 8 ? 2 : 3;
    int ct = 0, S = 0;
    rs_plan(w.N, w.K, M, Mtot, mod->part_floats, *S_io, &ct, &S);
    *S_io = S;
    const int groups = (n_tiles + ct - 1) / ct;
    if (rw == 2) switch (ct) {
        case 16: return launch_gemm_rs_t<16, 2>(w, act, plane, mtp, part, M, Mtot, S, groups, st);
        case 12: return launch_gemm_rs_t<12, 2>(w, act, plane, mtp, part, M, Mtot, S, groups, st);
        case 11: return launch_gemm_rs_t<11, 2>(w, act, plane, mtp, part, M, Mtot, S, groups, st);
        case 8: return launch_gemm_rs_t<8, 2>(w, act, plane, mtp, part, M, Mtot, S, groups, st);
        default: return launch_gemm_rs_t<6, 2>(w, act, plane, mtp, part, M, Mtot, S, groups, st);
    }
    if (MT <= 12) return ct == 8 ? launch_gemm_rs_t<8, 3>(w, act, plane, mtp, part, M, Mtot, S, groups, st)
                                : launch_gemm_rs_t<6, 3>(w, act, plane, mtp, part, M, Mtot, S, groups, st);
    return CSD_ESHAPE;
}

// Once per process and device, at model creation (no runtime call besides launches happens later): allow
// every GEMM instantiation its dynamic LDS (up to 144 KB).
template <int MT>
static hipError_t ws_allow_lds() {
    return hipFuncSetAttribute((const void *)k_gemm_ws<1, MT, WG_U_MAX>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               2 * WG_U_MAX * MT * 2 * 64 * 16);
}
template <int CT, int RW>
static hipError_t rs_allow_lds() {
    return hipFuncSetAttribute((const void *)k_gemm_rs<CT, RW, WG_U_MAX>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               2 * WG_U_MAX * CT * 64 * 16);
}
int32_t csd_gemm_setup() {
    CSD_HIP(ws_allow_lds<1>());
    CSD_HIP(ws_allow_lds<2>());
    CSD_HIP((rs_allow_lds<16, 2>()));
    CSD_HIP((rs_allow_lds<12, 2>()));
    CSD_HIP((rs_allow_lds<11, 2>()));
    CSD_HIP((rs_allow_lds<8, 2>()));
    CSD_HIP((rs_allow_lds<6, 2>()));
    CSD_HIP((rs_allow_lds<8, 3>()));
    CSD_HIP((rs_allow_lds<6, 3>()));
    return CSD_OK;
}

// act: M rows of width w.K in the path's activation form; part: [S][M][w.N] with S (<= w.S) returned in *S_used
static int32_t run_gemm(csd_model *mod, const GemmW &w, const void *act, int M, int *S_used, hipStream_t st) {
    ProfScope ps(mod, st, CSD_PROF_GEMM);
    *S_used = w.S;
    if (mod->mfma) {
        // up to 144 rows in one launch, more in chunks of 128 rows that share the number of K splits
        *S_used = 0;
        const int step = M <= 144 ? M : 128;
        for (int row0 = 0; row0 < M; row0 += step) {
            const int rows = M - row0 < step ? M - row0 : step;
            const bf16_t *a = (const bf16_t *)act + (size_t)(row0 / 16) * 512;   // row tile row0 / 16 of every k-step
            float *p = mod->part + (size_t)row0 * w.N;
            const int32_t rc = rows >= mod->gemm_rs_min_rows
                                   ? launch_gemm_rs(mod, w, a, mod->act_plane, mod->act_mtp, p, rows, M, S_used, st)
                                   : launch_gemm_ws(w, a, mod->act_plane, mod->act_mtp, p, rows, M, S_used, st);
            if (rc != CSD_OK) return rc;
        }
    } else if (mod->cfg.dtype == CSD_DTYPE_BF16) {
        hipLaunchKernelGGL((k_gemm_simple<bf16_t>), dim3((w.N + 255) / 256), dim3(256), 0, st, (const bf16_t *)w.data,
                           (const float *)act, mod->part, M, w.K, w.N);
    } else {
        hipLaunchKernelGGL((k_gemm_simple<float>), dim3((w.N + 255) / 256), dim3(256), 0, st, (const float *)w.data,
                           (const float *)act, mod->part, M, w.K, w.N);
    }
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

int32_t csd_attn_mfma_enqueue(csd_model *mod, const KvGeom &geo, const void *kv, const int32_t *cache_len, int B, int m,
                              int layer, float scale, const AttnMode &mode, hipStream_t st, bf16_t *out = nullptr,
                              size_t out_plane = 0);   // csd_attention.hip

template <typename TW, typename TA, typename TC>
static int32_t forward_typed(csd_model *mod, void *kv, const int32_t *tokens, const int32_t *cache_len, int32_t B,
                             int32_t m, float *logits, hipStream_t st) {
    const csd_model_cfg &c = mod->cfg;
    const int M = B * m, d = c.d_model, F = c.d_ffn, hd = mod->hd, V = c.vocab, L = c.n_layers;
    const KvGeom geo = geom(mod);
    TA *act = (TA *)mod->act;
    TA *qb = (TA *)mod->qbuf;
    const int lda = d > F ? (d > hd ? d : hd) : (F > hd ? F : hd);   // rows of `act` are reused at several widths
    (void)lda;
    const float scale = 1.0f / sqrtf((float)c.head_dim);
    int S_g = 1;            // K splits the last GEMM wrote partial sums for
    {
        ProfScope ps(mod, st, CSD_PROF_OTHER);
        hipLaunchKernelGGL((k_embed_norm<TW, TA>), dim3(M), dim3(256), 0, st, tokens, (const TW *)mod->embed, V, d,
                           mod->layers[0].attn_norm, c.rms_eps, mod->h, act, d, mod->act_plane, mod->act_mtp, mod->rstd);
        CSD_LAUNCH_CHECK();
    }
    if (mod->trace) CSD_HIP(hipMemcpyAsync(mod->trace, mod->h, sizeof(float) * (size_t)M * d, hipMemcpyDeviceToDevice, st));
    if (c.rope_theta > 0.f) {
        ProfScope ps(mod, st, CSD_PROF_OTHER);
        hipLaunchKernelGGL(k_rope_table, dim3(M), dim3(64), 0, st, cache_len, m, c.head_dim, c.rope_theta, mod->rope,
                           mod->tree_call ? mod->tree_depth : nullptr);
        CSD_LAUNCH_CHECK();
    }
    for (int l = 0; l < L; l++) {
        const LayerW &lw = mod->layers[l];
        int32_t rc;
        if ((rc = run_gemm(mod, lw.qkv, act, M, &S_g, st)) != CSD_OK) return rc;
        {
            ProfScope ps(mod, st, CSD_PROF_OTHER);
            hipLaunchKernelGGL((k_fix_qkv<TA, TC>), dim3(M, c.n_heads), dim3(64), 0, st, mod->part, S_g, M, m,
                               cache_len, geo, l, c.rope_theta > 0.f ? mod->rope : nullptr, qb, mod->q_plane, (TC *)kv, mod->rstd);
            CSD_LAUNCH_CHECK();
        }
        AttnMode am;
        if (mod->tree_call) am.anc = mod->tree_anc;
        if (mod->mfma_attn) {
            if ((rc = csd_attn_mfma_enqueue(mod, geo, kv, cache_len, B, m, l, scale, am, st)) != CSD_OK) return rc;
        } else {
            ProfScope ps(mod, st, CSD_PROF_ATTN);
            const size_t lds = sizeof(float) * (size_t)(c.head_dim + mod->seq_pad);
            hipLaunchKernelGGL((k_attn_simple<TA, TC>), dim3(M, c.n_heads), dim3(64), lds, st, qb, m, cache_len, geo, l,
                               (const TC *)kv, scale, mod->q_plane, act, hd, mod->act_plane, mod->act_mtp, am);
            CSD_LAUNCH_CHECK();
        }
        if ((rc = run_gemm(mod, lw.o, act, M, &S_g, st)) != CSD_OK) return rc;
        {
            ProfScope ps(mod, st, CSD_PROF_OTHER);
            hipLaunchKernelGGL((k_residual_norm<TA>), dim3(M), dim3(RN_THREADS), 0, st, mod->part, S_g, M, d, lw.ffn_norm,
                               c.rms_eps, mod->h, act, d, mod->act_plane, mod->act_mtp, mod->rstd);
            CSD_LAUNCH_CHECK();
        }
        if ((rc = run_gemm(mod, lw.gu, act, M, &S_g, st)) != CSD_OK) return rc;
        {
            ProfScope ps(mod, st, CSD_PROF_OTHER);
            hipLaunchKernelGGL((k_fix_gu<TA>), dim3((F + 255) / 256, M), dim3(256), 0, st, mod->part, S_g, M, F,
                               mod->mfma ? 1 : 0, act, F, mod->act_plane, mod->act_mtp, 0, mod->rstd);
            CSD_LAUNCH_CHECK();
        }
        if ((rc = run_gemm(mod, lw.down, act, M, &S_g, st)) != CSD_OK) return rc;
        {
            ProfScope ps(mod, st, CSD_PROF_OTHER);
            const float *g = (l + 1 < L) ? mod->layers[l + 1].attn_norm : mod->final_norm;
            hipLaunchKernelGGL((k_residual_norm<TA>), dim3(M), dim3(RN_THREADS), 0, st, mod->part, S_g, M, d, g,
                               c.rms_eps, mod->h, act, d, mod->act_plane, mod->act_mtp, mod->rstd);
            CSD_LAUNCH_CHECK();
        }
        if (mod->trace)
            CSD_HIP(hipMemcpyAsync(mod->trace + (size_t)(l + 1) * M * d, mod->h, sizeof(float) * (size_t)M * d,
                                   hipMemcpyDeviceToDevice, st));
    }
    int32_t rc;
    if ((rc = run_gemm(mod, mod->lm, act, M, &S_g, st)) != CSD_OK) return rc;
    {
        ProfScope ps(mod, st, CSD_PROF_OTHER);
        hipLaunchKernelGGL(k_fix_logits, dim3((V + 255) / 256, M), dim3(256), 0, st, mod->part, S_g, M, V, logits, mod->rstd);
        CSD_LAUNCH_CHECK();
    }
    return CSD_OK;
}

static KvGeom cross_geom(const csd_model *mod) {
    return KvGeom{mod->cfg.max_batch, mod->cfg.n_heads, mod->cfg.head_dim, mod->enc_pad, mod->cfg.n_layers, 0};
}

template <typename TA, typename TC>
static int32_t attention_any(csd_model *mod, const KvGeom &geo, const void *kvbase, const int32_t *cache_len, int B, int m,
                             int layer, float scale, const AttnMode &mode, hipStream_t st) {
    if (mod->mfma_attn) return csd_attn_mfma_enqueue(mod, geo, kvbase, cache_len, B, m, layer, scale, mode, st);
    ProfScope ps(mod, st, CSD_PROF_ATTN);
    const size_t lds = sizeof(float) * (size_t)(mod->cfg.head_dim + geo.seq_pad);
    hipLaunchKernelGGL((k_attn_simple<TA, TC>), dim3(B * m, mod->cfg.n_heads), dim3(64), lds, st, (const TA *)mod->qbuf, m,
                       cache_len, geo, layer, (const TC *)kvbase, scale, mod->q_plane, (TA *)mod->act, mod->hd, mod->act_plane,
                       mod->act_mtp, mode);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

// arch 1: T5-style decoder.  Per layer: self-attention (no rotary embedding, unscaled scores plus the
// bucketed relative-position bias), cross-attention over the projected encoder rows in the cache's second
// part (no mask, no bias), gated tanh-GELU feed-forward; each sub-layer is norm -> op -> residual add.
template <typename TW, typename TA, typename TC>
static int32_t forward_t5(csd_model *mod, void *kv, const int32_t *tokens, const int32_t *cache_len, int32_t B, int32_t m,
                          float *logits, hipStream_t st) {
    const csd_model_cfg &c = mod->cfg;
    const int M = B * m, d = c.d_model, F = c.d_ffn, hd = mod->hd, V = c.vocab, L = c.n_layers;
    const KvGeom geo = geom(mod), cgeo = cross_geom(mod);
    TA *act = (TA *)mod->act;
    TA *qb = (TA *)mod->qbuf;
    const void *kv_cross = (const char *)kv + csd_self_kv_bytes(mod);
    AttnMode self_mode, cross_mode;
    self_mode.rel_bias = mod->rel_bias;
    self_mode.bucket = mod->rel_bucket;
    self_mode.bias_hd = mod->rel_bias_hd;
    cross_mode.fixed_nk = c.enc_len;
    int32_t rc;
    int S_g = 1;            // K splits the last GEMM wrote partial sums for
    auto resid_norm = [&](const GemmW &, const float *gain) -> int32_t {
        ProfScope ps(mod, st, CSD_PROF_OTHER);
        hipLaunchKernelGGL((k_residual_norm<TA>), dim3(M), dim3(RN_THREADS), 0, st, mod->part, S_g, M, d, gain, c.rms_eps, mod->h, act,
                           d, mod->act_plane, mod->act_mtp, mod->rstd);
        CSD_LAUNCH_CHECK();
        return CSD_OK;
    };
    {
        ProfScope ps(mod, st, CSD_PROF_OTHER);
        hipLaunchKernelGGL((k_embed_norm<TW, TA>), dim3(M), dim3(256), 0, st, tokens, (const TW *)mod->embed, V, d,
                           mod->layers[0].attn_norm, c.rms_eps, mod->h, act, d, mod->act_plane, mod->act_mtp, mod->rstd);
        CSD_LAUNCH_CHECK();
    }
    if (mod->trace) CSD_HIP(hipMemcpyAsync(mod->trace, mod->h, sizeof(float) * (size_t)M * d, hipMemcpyDeviceToDevice, st));
    for (int l = 0; l < L; l++) {
        const LayerW &lw = mod->layers[l];
        if ((rc = run_gemm(mod, lw.qkv, act, M, &S_g, st)) != CSD_OK) return rc;
        {
            ProfScope ps(mod, st, CSD_PROF_OTHER);
            hipLaunchKernelGGL((k_fix_qkv<TA, TC>), dim3(M, c.n_heads), dim3(64), 0, st, mod->part, S_g, M, m, cache_len,
                               geo, l, (const float2 *)nullptr, qb, mod->q_plane, (TC *)kv, mod->rstd);
            CSD_LAUNCH_CHECK();
        }
        if ((rc = attention_any<TA, TC>(mod, geo, kv, cache_len, B, m, l, 1.0f, self_mode, st)) != CSD_OK) return rc;
        if ((rc = run_gemm(mod, lw.o, act, M, &S_g, st)) != CSD_OK) return rc;
        if ((rc = resid_norm(lw.o, lw.cross_norm)) != CSD_OK) return rc;
        if ((rc = run_gemm(mod, lw.cq, act, M, &S_g, st)) != CSD_OK) return rc;
        {
            ProfScope ps(mod, st, CSD_PROF_OTHER);
            hipLaunchKernelGGL((k_fix_plain<TA>), dim3((hd + 255) / 256, M), dim3(256), 0, st, mod->part, S_g, M, hd, qb, hd,
                               mod->q_plane, mod->rstd);
            CSD_LAUNCH_CHECK();
        }
        if ((rc = attention_any<TA, TC>(mod, cgeo, kv_cross, cache_len, B, m, l, 1.0f, cross_mode, st)) != CSD_OK) return rc;
        if ((rc = run_gemm(mod, lw.co, act, M, &S_g, st)) != CSD_OK) return rc;
        if ((rc = resid_norm(lw.co, lw.ffn_norm)) != CSD_OK) return rc;
        if ((rc = run_gemm(mod, lw.gu, act, M, &S_g, st)) != CSD_OK) return rc;
        {
            ProfScope ps(mod, st, CSD_PROF_OTHER);
            hipLaunchKernelGGL((k_fix_gu<TA>), dim3((F + 255) / 256, M), dim3(256), 0, st, mod->part, S_g, M, F,
                               mod->mfma ? 1 : 0, act, F, mod->act_plane, mod->act_mtp, 1, mod->rstd);
            CSD_LAUNCH_CHECK();
        }
        if ((rc = run_gemm(mod, lw.down, act, M, &S_g, st)) != CSD_OK) return rc;
        if ((rc = resid_norm(lw.down, (l + 1 < L) ? mod->layers[l + 1].attn_norm : mod->final_norm)) != CSD_OK) return rc;
        if (mod->trace)
            CSD_HIP(hipMemcpyAsync(mod->trace + (size_t)(l + 1) * M * d, mod->h, sizeof(float) * (size_t)M * d,
                                   hipMemcpyDeviceToDevice, st));
    }
    if ((rc = run_gemm(mod, mod->lm, act, M, &S_g, st)) != CSD_OK) return rc;
    {
        ProfScope ps(mod, st, CSD_PROF_OTHER);
        hipLaunchKernelGGL(k_fix_logits, dim3((V + 255) / 256, M), dim3(256), 0, st, mod->part, S_g, M, V, logits, mod->rstd);
        CSD_LAUNCH_CHECK();
    }
    return CSD_OK;
}

// arch 1: project the encoder output of B sequences to every layer's cross-attention keys and values.
template <typename TA, typename TC>
static int32_t cross_init_typed(csd_model *mod, void *kv, const float *enc_out, int32_t B, hipStream_t st) {
    const csd_model_cfg &c = mod->cfg;
    const int d = c.d_model, hd = mod->hd, E = c.enc_len;
    const KvGeom cgeo = cross_geom(mod);
    TC *kvc = (TC *)((char *)kv + csd_self_kv_bytes(mod));
    const int chunk = mod->m_max;       // the activation and partial-sum buffers hold this many rows
    int32_t rc;
    int S_g = 1;
    for (int b = 0; b < B; b++)
        for (int row0 = 0; row0 < E; row0 += chunk) {
            const int rows = E - row0 < chunk ? E - row0 : chunk;
            {
                ProfScope ps(mod, st, CSD_PROF_OTHER);
                const size_t total = (size_t)rows * d;
                hipLaunchKernelGGL((k_rows_to_act<TA>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                                   enc_out + ((size_t)b * E + row0) * d, rows, d, (TA *)mod->act, d, mod->act_plane, mod->act_mtp);
                CSD_LAUNCH_CHECK();
            }
            for (int l = 0; l < c.n_layers; l++) {
                const LayerW &lw = mod->layers[l];
                if ((rc = run_gemm(mod, lw.ckv, mod->act, rows, &S_g, st)) != CSD_OK) return rc;
                ProfScope ps(mod, st, CSD_PROF_OTHER);
                hipLaunchKernelGGL((k_fix_cross_kv<TC>), dim3((hd + 255) / 256, rows), dim3(256), 0, st, mod->part, S_g, rows,
                                   cgeo, l, b, row0, kvc);
                CSD_LAUNCH_CHECK();
            }
        }
    return CSD_OK;
}

extern "C" int32_t csd_cross_kv_init(csd_model *mod, void *kv, const float *enc_out, int32_t B, void *stream) {
    if (!mod || !kv || !enc_out) return CSD_ENULL;
    if (mod->cfg.arch != 1) return CSD_EUNSUPPORTED;
    if (B < 1) return CSD_EINVAL;
    if (B > mod->cfg.max_batch) return CSD_ESHAPE;
    hipStream_t st = (hipStream_t)stream;
    if (mod->cfg.dtype == CSD_DTYPE_FP32) return cross_init_typed<float, float>(mod, kv, enc_out, B, st);
    if (mod->mfma) return cross_init_typed<bf16_t, bf16_t>(mod, kv, enc_out, B, st);
    return cross_init_typed<float, bf16_t>(mod, kv, enc_out, B, st);
}

int32_t csd_forward_enqueue(csd_model *mod, void *kv, const int32_t *tokens, const int32_t *cache_len, int32_t B,
                            int32_t m, float *logits, hipStream_t st) {
    if (csd_chain_eligible(mod, B, m)) return csd_chain_enqueue(mod, kv, tokens, cache_len, B, m, logits, st);
    if (mod->cfg.arch == 1) {
        if (mod->cfg.dtype == CSD_DTYPE_FP32) return forward_t5<float, float, float>(mod, kv, tokens, cache_len, B, m, logits, st);
        if (mod->mfma) return forward_t5<bf16_t, bf16_t, bf16_t>(mod, kv, tokens, cache_len, B, m, logits, st);
        return forward_t5<bf16_t, float, bf16_t>(mod, kv, tokens, cache_len, B, m, logits, st);
    }
    if (mod->cfg.dtype == CSD_DTYPE_FP32)
        return forward_typed<float, float, float>(mod, kv, tokens, cache_len, B, m, logits, st);
    if (mod->mfma) return forward_typed<bf16_t, bf16_t, bf16_t>(mod, kv, tokens, cache_len, B, m, logits, st);
    return forward_typed<bf16_t, float, bf16_t>(mod, kv, tokens, cache_len, B, m, logits, st);
}

// --------------------------------------------------------------------------- model building

static int pick_splits(int n_groups, int KS) {
    // enough waves to cover 256 CUs several times over, slices of at least 8 k-steps
    int S = 1;
    while (n_groups * S < 2048 && KS / (S * 2) >= 8 && S < 16) S *= 2;
    return S;
}

template <typename T>
static int32_t copy_cols(const void *src, int K, int N_src, void *dst, int N_dst, int col0, hipStream_t st) {
    const size_t total = (size_t)K * N_src;
    hipLaunchKernelGGL((k_copy_cols<T>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const T *)src, K, N_src,
                       (T *)dst, N_dst, col0);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

static int32_t pack_tiles(const void *src, int K, int N_src, void *dst, int base, int stride, int perm_dh,
                          hipStream_t st) {
    const size_t total = (size_t)(N_src / 16) * (K / 32) * 64;
    hipLaunchKernelGGL(k_pack_tiles, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const bf16_t *)src, K, N_src,
                       (bf16_t *)dst, K / 32, base, stride, perm_dh);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

static int32_t dev_alloc(csd_model *mod, void **p, size_t bytes) {
    CSD_HIP(hipMalloc(p, bytes ? bytes : 256));
    mod->allocs.push_back(*p);
    return CSD_OK;
}

struct Piece {
    const void *src;
    int N_src;
    int base, stride;   // tile placement (MFMA) ; col0 = base*16 (row-major)
    int perm_dh;        // > 0: take the piece's output features in rotary pair order (q and k projections)
};

static int32_t build_gemm(csd_model *mod, GemmW *g, int K, int N, const Piece *pieces, int n_pieces, bool interleave,
                          hipStream_t st) {
    const size_t esz = mod->cfg.dtype == CSD_DTYPE_BF16 ? 2 : 4;
    g->K = K;
    g->N = N;
    int32_t rc;
    if ((rc = dev_alloc(mod, &g->data, (size_t)K * N * esz)) != CSD_OK) return rc;
    if (mod->mfma) {
        g->S = pick_splits(N / 16, K / 32);
        for (int i = 0; i < n_pieces; i++)
            if ((rc = pack_tiles(pieces[i].src, K, pieces[i].N_src, g->data, pieces[i].base, pieces[i].stride,
                                 mod->kperm ? pieces[i].perm_dh : 0, st)) != CSD_OK)
                return rc;
    } else {
        g->S = 1;
        (void)interleave;
        int col0 = 0;
        for (int i = 0; i < n_pieces; i++) {
            if (esz == 2)
                rc = copy_cols<bf16_t>(pieces[i].src, K, pieces[i].N_src, g->data, N, col0, st);
            else
                rc = copy_cols<float>(pieces[i].src, K, pieces[i].N_src, g->data, N, col0, st);
            if (rc != CSD_OK) return rc;
            col0 += pieces[i].N_src;
        }
    }
    if (g->S > mod->s_max) mod->s_max = g->S;
    return CSD_OK;
}

int32_t csd_pack_weights(csd_model *mod, const void *const *w, hipStream_t st) {
    const csd_model_cfg &c = mod->cfg;
    const int d = c.d_model, F = c.d_ffn, hd = mod->hd, V = c.vocab, L = c.n_layers;
    const size_t esz = c.dtype == CSD_DTYPE_BF16 ? 2 : 4;
    int32_t rc;
    if ((rc = dev_alloc(mod, &mod->embed, (size_t)V * d * esz)) != CSD_OK) return rc;
    CSD_HIP(hipMemcpyAsync(mod->embed, w[0], (size_t)V * d * esz, hipMemcpyDeviceToDevice, st));
    mod->layers.resize(L);
    if (c.arch == 1) {
        // canonical order per layer: self_norm, wq, wk, wv, wo, cross_norm, cq, ck, cv, co, ffn_norm, w0, w1, w_out;
        // then final_norm, lm_head, rel_bias [32][H] fp32
        for (int l = 0; l < L; l++) {
            const void *const *lw = w + 1 + 14 * l;
            LayerW &o = mod->layers[l];
            float **norms[3] = {&o.attn_norm, &o.cross_norm, &o.ffn_norm};
            const int norm_idx[3] = {0, 5, 10};
            for (int i = 0; i < 3; i++) {
                if ((rc = dev_alloc(mod, (void **)norms[i], sizeof(float) * d)) != CSD_OK) return rc;
                CSD_HIP(hipMemcpyAsync(*norms[i], lw[norm_idx[i]], sizeof(float) * d, hipMemcpyDeviceToDevice, st));
            }
            const Piece qkv[3] = {{lw[1], hd, 0, 1, 0}, {lw[2], hd, hd / 16, 1, 0}, {lw[3], hd, 2 * hd / 16, 1, 0}};
            if ((rc = build_gemm(mod, &o.qkv, d, 3 * hd, qkv, 3, false, st)) != CSD_OK) return rc;
            const Piece wo[1] = {{lw[4], d, 0, 1, 0}};
            if ((rc = build_gemm(mod, &o.o, hd, d, wo, 1, false, st)) != CSD_OK) return rc;
            const Piece cq[1] = {{lw[6], hd, 0, 1, 0}};
            if ((rc = build_gemm(mod, &o.cq, d, hd, cq, 1, false, st)) != CSD_OK) return rc;
            const Piece ckv[2] = {{lw[7], hd, 0, 1, 0}, {lw[8], hd, hd / 16, 1, 0}};
            if ((rc = build_gemm(mod, &o.ckv, d, 2 * hd, ckv, 2, false, st)) != CSD_OK) return rc;
            const Piece co[1] = {{lw[9], d, 0, 1, 0}};
            if ((rc = build_gemm(mod, &o.co, hd, d, co, 1, false, st)) != CSD_OK) return rc;
            const Piece gu[2] = {{lw[11], F, 0, 2, 0}, {lw[12], F, 1, 2, 0}};
            if ((rc = build_gemm(mod, &o.gu, d, 2 * F, gu, 2, true, st)) != CSD_OK) return rc;
            const Piece dn[1] = {{lw[13], d, 0, 1, 0}};
            if ((rc = build_gemm(mod, &o.down, F, d, dn, 1, false, st)) != CSD_OK) return rc;
        }
        if ((rc = dev_alloc(mod, (void **)&mod->final_norm, sizeof(float) * d)) != CSD_OK) return rc;
        CSD_HIP(hipMemcpyAsync(mod->final_norm, w[1 + 14 * L], sizeof(float) * d, hipMemcpyDeviceToDevice, st));
        const Piece lm[1] = {{w[2 + 14 * L], V, 0, 1, 0}};
        if ((rc = build_gemm(mod, &mod->lm, d, V, lm, 1, false, st)) != CSD_OK) return rc;
        if ((rc = dev_alloc(mod, (void **)&mod->rel_bias, sizeof(float) * 32 * c.n_heads)) != CSD_OK) return rc;
        CSD_HIP(hipMemcpyAsync(mod->rel_bias, w[3 + 14 * L], sizeof(float) * 32 * c.n_heads, hipMemcpyDeviceToDevice, st));
        // bucket of a look-back distance n (T5's unidirectional scheme with 32 buckets, maximum distance 128):
        // n itself below 16, then 16 logarithmically spaced buckets up to 128, farther keys in the last one
        int32_t tab[128];
        for (int n = 0; n < 128; n++) {
            int bkt = n;
            if (n >= 16) {
                bkt = 16 + (int)(std::log((double)n / 16.0) / std::log(128.0 / 16.0) * 16.0);
                if (bkt > 31) bkt = 31;
            }
            tab[n] = bkt;
        }
        tab[127] = 31;
        if ((rc = dev_alloc(mod, (void **)&mod->rel_bucket, sizeof(tab))) != CSD_OK) return rc;
        CSD_HIP(hipMemcpy(mod->rel_bucket, tab, sizeof(tab), hipMemcpyHostToDevice));
        if ((rc = dev_alloc(mod, (void **)&mod->rel_bias_hd, sizeof(float) * 128 * c.n_heads)) != CSD_OK) return rc;
        hipLaunchKernelGGL(k_bias_table, dim3(c.n_heads), dim3(128), 0, st, mod->rel_bias, mod->rel_bucket, c.n_heads, mod->rel_bias_hd);
        CSD_LAUNCH_CHECK();
        return CSD_OK;
    }
    for (int l = 0; l < L; l++) {
        const void *const *lw = w + 1 + 9 * l;
        LayerW &o = mod->layers[l];
        if ((rc = dev_alloc(mod, (void **)&o.attn_norm, sizeof(float) * d)) != CSD_OK) return rc;
        if ((rc = dev_alloc(mod, (void **)&o.ffn_norm, sizeof(float) * d)) != CSD_OK) return rc;
        CSD_HIP(hipMemcpyAsync(o.attn_norm, lw[0], sizeof(float) * d, hipMemcpyDeviceToDevice, st));
        CSD_HIP(hipMemcpyAsync(o.ffn_norm, lw[5], sizeof(float) * d, hipMemcpyDeviceToDevice, st));
        const Piece qkv[3] = {{lw[1], hd, 0, 1, c.head_dim}, {lw[2], hd, hd / 16, 1, c.head_dim}, {lw[3], hd, 2 * hd / 16, 1, 0}};
        if ((rc = build_gemm(mod, &o.qkv, d, 3 * hd, qkv, 3, false, st)) != CSD_OK) return rc;
        const Piece wo[1] = {{lw[4], d, 0, 1, 0}};
        if ((rc = build_gemm(mod, &o.o, hd, d, wo, 1, false, st)) != CSD_OK) return rc;
        const Piece gu[2] = {{lw[6], F, 0, 2, 0}, {lw[7], F, 1, 2, 0}};
        if ((rc = build_gemm(mod, &o.gu, d, 2 * F, gu, 2, true, st)) != CSD_OK) return rc;
        const Piece dn[1] = {{lw[8], d, 0, 1, 0}};
        if ((rc = build_gemm(mod, &o.down, F, d, dn, 1, false, st)) != CSD_OK) return rc;
    }
    if ((rc = dev_alloc(mod, (void **)&mod->final_norm, sizeof(float) * d)) != CSD_OK) return rc;
    CSD_HIP(hipMemcpyAsync(mod->final_norm, w[1 + 9 * L], sizeof(float) * d, hipMemcpyDeviceToDevice, st));
    const Piece lm[1] = {{w[2 + 9 * L], V, 0, 1, 0}};
    if ((rc = build_gemm(mod, &mod->lm, d, V, lm, 1, false, st)) != CSD_OK) return rc;
    return CSD_OK;
}

// ------------------------------------------------------------------------------ cache access

size_t csd_self_kv_bytes(const csd_model *mod) {
    const csd_model_cfg &c = mod->cfg;
    const size_t esz = c.dtype == CSD_DTYPE_BF16 ? 2 : 4;
    return (size_t)2 * c.n_layers * c.max_batch * c.n_heads * mod->seq_pad * c.head_dim * esz;
}

extern "C" size_t csd_kv_bytes(const csd_model *mod) {
    if (!mod) return 0;
    const csd_model_cfg &c = mod->cfg;
    const size_t esz = c.dtype == CSD_DTYPE_BF16 ? 2 : 4;
    // arch 1 appends the cross-attention keys and values of every layer (filled by csd_cross_kv_init)
    const size_t cross = c.arch == 1 ? (size_t)2 * c.n_layers * c.max_batch * c.n_heads * mod->enc_pad * c.head_dim * esz : 0;
    return csd_self_kv_bytes(mod) + cross;
}

extern "C" int32_t csd_kv_write(const csd_model *mod, void *kv, int32_t layer, int32_t b, int32_t pos0, int32_t n,
                                const float *K, const float *V, void *stream) {
    if (!mod || !kv || !K || !V) return CSD_ENULL;
    const csd_model_cfg &c = mod->cfg;
    if (layer < 0 || layer >= c.n_layers || b < 0 || b >= c.max_batch || pos0 < 0 || n < 0) return CSD_EINVAL;
    if (pos0 + n > c.max_seq) return CSD_ESHAPE;
    if (n == 0) return CSD_OK;
    const size_t total = (size_t)n * mod->hd;
    const dim3 grid((unsigned)((total + 255) / 256));
    if (c.dtype == CSD_DTYPE_BF16)
        hipLaunchKernelGGL((k_kv_write<bf16_t>), grid, dim3(256), 0, (hipStream_t)stream, (bf16_t *)kv, geom(mod), layer, b,
                           pos0, n, K, V);
    else
        hipLaunchKernelGGL((k_kv_write<float>), grid, dim3(256), 0, (hipStream_t)stream, (float *)kv, geom(mod), layer, b,
                           pos0, n, K, V);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

extern "C" int32_t csd_kv_read(const csd_model *mod, const void *kv, int32_t layer, int32_t b, int32_t pos0, int32_t n,
                               float *K, float *V, void *stream) {
    if (!mod || !kv || !K || !V) return CSD_ENULL;
    const csd_model_cfg &c = mod->cfg;
    if (layer < 0 || layer >= c.n_layers || b < 0 || b >= c.max_batch || pos0 < 0 || n < 0) return CSD_EINVAL;
    if (pos0 + n > c.max_seq) return CSD_ESHAPE;
    if (n == 0) return CSD_OK;
    const size_t total = (size_t)n * mod->hd;
    const dim3 grid((unsigned)((total + 255) / 256));
    if (c.dtype == CSD_DTYPE_BF16)
        hipLaunchKernelGGL((k_kv_read<bf16_t>), grid, dim3(256), 0, (hipStream_t)stream, (const bf16_t *)kv, geom(mod), layer,
                           b, pos0, n, K, V);
    else
        hipLaunchKernelGGL((k_kv_read<float>), grid, dim3(256), 0, (hipStream_t)stream, (const float *)kv, geom(mod), layer, b,
                           pos0, n, K, V);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}
