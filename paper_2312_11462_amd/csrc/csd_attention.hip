// Causal block attention of the drafted block over the cached prefix, on the matrix cores.
//
// One wave per (sequence, head, chunk of 128 or more keys, 16-row tile of the block).  Both contractions
// are written transposed so that no operand ever needs a shuffle through LDS:
//   S^T = K * q^T   A = K rows (16 keys x 32 of dh), B = q (32 of dh x 16 block rows)
//   O^T = V^T * P^T A = V^T (16 of dh x 32 keys),     B = P^T (32 keys x 16 block rows)
// The result layout of the first product (lane = block row, 4 consecutive A-rows per register
// group) becomes the B operand of the second directly, because the keys are assigned to A-rows
// so that every lane ends up holding 8 consecutive keys; V is cached transposed so that the
// matching A operand is one 16-byte load.  Chunks keep an online-softmax state (max, sum,
// un-normalised output) that a small merge kernel combines.  The host doubles the keys per wave
// (chunk_keys) while there are more than two waves per SIMD, which shrinks the partial states the merge
// kernel has to read.  (A form that loads each key tile once for two row tiles of
// the block was slower: its register need halves the waves in flight.)
#include "csd_internal.h"

#define ATT_CHUNK 128      /* keys per wave at least (the partial buffer is sized for this) */

// ONCE: this launch reads every cache row once (one 16-row tile per sequence), so the rows are loaded non-temporally and
// do not push each other out of the caches on their way through (batch 8 over 2048 rows: 55.7 -> 51.4 us per layer);
// with more row tiles the later passes find part of the rows in the caches and plain loads are kept.
template <bool ONCE>
__device__ __forceinline__ u32x4 attn_load(const bf16_t *p) {
    if constexpr (ONCE) return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    else return *reinterpret_cast<const u32x4 *>(p);
}

// PRE: key tiles (32 keys) whose K and V fragments are requested together before any of them is used.
// A small grid (few sequences and heads) is bound by the chain of memory round trips of each wave, not by
// bandwidth: with PRE = 4 a wave has its whole 128-key chunk in flight at once (at the price of registers,
// i.e. of waves per SIMD, which such a grid does not fill anyway).
template <int DH, int PRE, bool ONCE>
__global__ __launch_bounds__(64) void k_attn_mfma(const bf16_t *__restrict__ q, size_t qplane, int m, int row_tiles,
                                                  const int32_t *__restrict__ cache_len, KvGeom geo, int layer,
                                                  const bf16_t *__restrict__ kv, float scale, float *__restrict__ part,
                                                  int chunks_max, int chunk_keys, AttnMode mode) {
    constexpr int PS = DH + 4;   // floats per partial row: DH outputs, running max, running sum, pad
    // the chunk index is the slowest grid dimension: the last chunk of every (sequence, head) holds the block's own few
    // rows and little else, and with those short waves dispatched last the long ones land one per SIMD, four per
    // compute unit (dispatched every fifth, they left one SIMD of most compute units with two long waves and one with none)
    const int hh = blockIdx.x, b = blockIdx.y / row_tiles, rt = blockIdx.y % row_tiles, c = blockIdx.z;
    const int lane = threadIdx.x, col = lane & 15, g = lane >> 4;
    const int hd = geo.H * DH;
    const bool causal = mode.fixed_nk <= 0;
    const int t = causal ? cache_len[b] : 0;
    const int nk = max(0, min(causal ? t + m : mode.fixed_nk, geo.seq_pad));   // cache rows in play for this block
    float *po = part + ((((size_t)b * geo.H + hh) * chunks_max + c) * row_tiles + rt) * 16 * PS;
    float *pr = po + (size_t)col * PS;
    const int key0 = c * chunk_keys;
    if (key0 >= nk) {                                        // chunk past the end: neutral element
        if (g == 0) {
            pr[DH] = -INFINITY;
            pr[DH + 1] = 0.f;
        }
        return;
    }
    const int row = rt * 16 + col;                           // this lane's block row
    const int qpos = t + row;                                // it sees cache rows 0..qpos
    const unsigned long long anc_row = (mode.anc && row < m) ? mode.anc[b * m + row] : 0ull;
    u32x4 qf[DH / 32][2];                                    // hi and lo planes of the query
#pragma unroll
    for (int s = 0; s < DH / 32; s++) {
        qf[s][0] = qf[s][1] = u32x4{0u, 0u, 0u, 0u};
        if (row < m) {
            const bf16_t *qp = q + (size_t)(b * m + row) * hd + hh * DH + s * 32 + 8 * g;
            qf[s][0] = *reinterpret_cast<const u32x4 *>(qp);
            qf[s][1] = *reinterpret_cast<const u32x4 *>(qp + qplane);
        }
    }
    const bf16_t *kc = kv + kv_k_off(geo, layer, b, hh);
    const bf16_t *vc = kv + kv_v_off(geo, layer, b, hh);

    f32x4 oacc[DH / 16];
#pragma unroll
    for (int dt = 0; dt < DH / 16; dt++) oacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float mrun = -INFINITY, lrun = 0.f;

    for (int sub0 = 0; sub0 < chunk_keys / 32; sub0 += PRE) {
        if (key0 + sub0 * 32 >= nk) break;
        // A operands of PRE tiles.  K: A-row r of tile T is key kb + 8*(r/4) + 4*T + r%4, so lane group g ends up
        // with the scores of keys kb+8g..kb+8g+7; V^T: row = feature dt*16 + col, 8 consecutive keys per lane.
        u32x4 kf[PRE][2][DH / 32], vfr[PRE][DH / 16];
        float bias[PRE][8];                                  // relative-position bias of this lane's 8 keys per tile
#pragma unroll
        for (int p = 0; p < PRE; p++) {
            const int kb = key0 + (sub0 + p) * 32;
#pragma unroll
            for (int j = 0; j < 8; j++) bias[p][j] = 0.f;
            if (mode.bias_hd && kb < nk && sub0 + p < chunk_keys / 32) {     // uniform; fetched with the tile, ahead of its scores
#pragma unroll
                for (int j = 0; j < 8; j++)
                    bias[p][j] = mode.bias_hd[hh * 128 + min(max(qpos - (kb + 8 * g + j), 0), 127)];
            }
            if (kb < nk && sub0 + p < chunk_keys / 32) {     // uniform
#pragma unroll
                for (int T = 0; T < 2; T++) {
                    const int key = kb + 8 * (col >> 2) + 4 * T + (col & 3);
                    const bf16_t *kp = kc + (size_t)key * DH + 8 * g;
#pragma unroll
                    for (int s = 0; s < DH / 32; s++) kf[p][T][s] = attn_load<ONCE>(kp + s * 32);
                }
#pragma unroll
                for (int dt = 0; dt < DH / 16; dt++)
                    vfr[p][dt] = attn_load<ONCE>(vc + kv_v_idx(geo, dt * 16 + col, kb + 8 * g));
            } else {
#pragma unroll
                for (int T = 0; T < 2; T++)
#pragma unroll
                    for (int s = 0; s < DH / 32; s++) kf[p][T][s] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
                for (int dt = 0; dt < DH / 16; dt++) vfr[p][dt] = u32x4{0u, 0u, 0u, 0u};
            }
        }
#pragma unroll
        for (int p = 0; p < PRE; p++) {
            const int kb = key0 + (sub0 + p) * 32;
            if (kb >= nk || sub0 + p >= chunk_keys / 32) break;
            f32x4 sT[2];
#pragma unroll
            for (int T = 0; T < 2; T++) {
                sT[T] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < DH / 32; s++) {
                    sT[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[p][T][s]),
                                                                    __builtin_bit_cast(bf16x8, qf[s][0]), sT[T], 0, 0, 0);
                    sT[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[p][T][s]),
                                                                    __builtin_bit_cast(bf16x8, qf[s][1]), sT[T], 0, 0, 0);
                }
            }
            float sv[8];
            float mx = -INFINITY;
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const int key = kb + 8 * g + j;
                float s = sT[j >> 2][j & 3] * scale;
                const bool seen = (mode.anc ? tree_sees(anc_row, key, t) : (!causal || key <= qpos)) && key < nk;
                s += bias[p][j];                             // 0 without a bias table; unseen keys are masked next
                sv[j] = seen ? s : -INFINITY;
                mx = fmaxf(mx, sv[j]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float mnew = fmaxf(mrun, mx);
            const float alpha = (mnew == -INFINITY) ? 1.0f : expf(mrun - mnew);
            float pv[8];
            float psum = 0.f;
#pragma unroll
            for (int j = 0; j < 8; j++) {
                pv[j] = (sv[j] == -INFINITY) ? 0.f : expf(sv[j] - mnew);
                psum += pv[j];
            }
            psum += __shfl_xor(psum, 16, 64);
            psum += __shfl_xor(psum, 32, 64);
            lrun = lrun * alpha + psum;
            mrun = mnew;
            u32x4 pf, pl;                                    // hi and lo planes of the probabilities
#pragma unroll
            for (int w = 0; w < 4; w++) {
                const bf16_t h0 = f32_to_bf16(pv[2 * w]), h1 = f32_to_bf16(pv[2 * w + 1]);
                pf[w] = (uint32_t)h0 | ((uint32_t)h1 << 16);
                pl[w] = (uint32_t)f32_to_bf16(pv[2 * w] - bf16_to_f32(h0)) |
                        ((uint32_t)f32_to_bf16(pv[2 * w + 1] - bf16_to_f32(h1)) << 16);
            }
            const bool tail = kb + 32 > nk;                  // rows past nk may hold anything: zero them
#pragma unroll
            for (int dt = 0; dt < DH / 16; dt++) {
                u32x4 vf = vfr[p][dt];
                if (tail) {
#pragma unroll
                    for (int w = 0; w < 4; w++) {
                        const int k0 = kb + 8 * g + 2 * w;
                        const uint32_t keep = (k0 < nk ? 0x0000FFFFu : 0u) | (k0 + 1 < nk ? 0xFFFF0000u : 0u);
                        vf[w] &= keep;
                    }
                }
                oacc[dt] = oacc[dt] * alpha;
                oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf),
                                                                   __builtin_bit_cast(bf16x8, pf), oacc[dt], 0, 0, 0);
                oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf),
                                                                   __builtin_bit_cast(bf16x8, pl), oacc[dt], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int dt = 0; dt < DH / 16; dt++) *reinterpret_cast<f32x4 *>(pr + dt * 16 + 4 * g) = oacc[dt];
    if (g == 0) {
        pr[DH] = mrun;
        pr[DH + 1] = lrun;
    }
}

// out[r][hh*DH + x] = sum_c acc_c[x] e^(m_c - m*) / sum_c l_c e^(m_c - m*)
template <int DH>
__global__ __launch_bounds__(DH) void k_attn_merge(const float *__restrict__ part, int m, int row_tiles,
                                                   const int32_t *__restrict__ cache_len, int H, int seq_pad,
                                                   int chunks_max, int chunk_keys, bf16_t *__restrict__ out, int ldo,
                                                   size_t plane, int mtp, int fixed_nk) {
    constexpr int PS = DH + 4;
    const int r = blockIdx.x, hh = blockIdx.y, x = threadIdx.x;
    const int b = r / m, i = r % m, rt = i / 16, ri = i % 16;
    const int nk = max(1, min(fixed_nk > 0 ? fixed_nk : cache_len[b] + m, seq_pad));
    const int nch = (nk + chunk_keys - 1) / chunk_keys;
    const float *base = part + (((size_t)b * H + hh) * chunks_max * row_tiles + rt) * 16 * PS + (size_t)ri * PS;
    const size_t cstride = (size_t)row_tiles * 16 * PS;
    // chunk states are read eight at a time (the index is clamped rather than the load skipped, so all eight
    // loads are in flight together) and folded in chunk order with a running maximum: one pass over the
    // states, one memory round trip per eight chunks
    float mstar = -INFINITY, num = 0.f, den = 0.f;
    for (int c0 = 0; c0 < nch; c0 += 8) {
        float mc[8], ac[8], lc[8];
#pragma unroll
        for (int u = 0; u < 8; u++) {
            const size_t o = (size_t)min(c0 + u, nch - 1) * cstride;
            mc[u] = base[o + DH];
            ac[u] = base[o + x];
            lc[u] = base[o + DH + 1];
        }
        float mnew = mstar;
#pragma unroll
        for (int u = 0; u < 8; u++)
            if (c0 + u < nch) mnew = fmaxf(mnew, mc[u]);
        const float a = (mstar == -INFINITY) ? 0.f : expf(mstar - mnew);
        num *= a;
        den *= a;
#pragma unroll
        for (int u = 0; u < 8; u++) {
            if (c0 + u >= nch || mc[u] == -INFINITY) continue;
            const float w = expf(mc[u] - mnew);
            num += ac[u] * w;
            den += lc[u] * w;
        }
        mstar = mnew;
    }
    store_act<bf16_t>(out, plane, r, hh * DH + x, ldo, mtp, den > 0.f ? num / den : 0.f);
}

template <int DH>
static void attn_launch(csd_model *mod, const KvGeom &geo, const void *kv, const int32_t *cache_len, int B, int m, int layer,
                        float scale, const AttnMode &mode, hipStream_t st, bf16_t *out, size_t out_plane) {
    const csd_model_cfg &c = mod->cfg;
    const int row_tiles = (m + 15) / 16;
    // Keys per wave.  The kernel's registers allow two waves per SIMD, and waves beyond 2048 would wait for a second
    // round: chunks of 128 keys when that many waves fit; otherwise as many equal chunks per (sequence, head, row tile)
    // as fit, of at least 512 keys (measured at batch 8 with 2048 cached rows, one row tile: 1.88 ms of attention per
    // step with 4 to 6 chunks per head against 2.04 with 8; two row tiles: 2.40 ms with 4 equal chunks against 2.91
    // with two of 1024 keys and a short third).
    const int keys = mode.fixed_nk > 0 ? mode.fixed_nk : geo.seq_pad;
    const long long items = (long long)c.n_heads * B * row_tiles;
    const int n_max = (keys + ATT_CHUNK - 1) / ATT_CHUNK;
    int n_c = (int)(2048 / items < n_max ? 2048 / items : n_max);
    if (n_c < n_max && n_c > keys / 512) n_c = keys / 512;
    if (n_c < 1) n_c = 1;
    const int chunk_keys = n_c == n_max ? ATT_CHUNK : ((keys + n_c - 1) / n_c + 31) / 32 * 32;
    int chunks = (keys + chunk_keys - 1) / chunk_keys;
    if (chunks > mod->attn_chunks_max) chunks = mod->attn_chunks_max;
    // a grid the chip holds at one wave per SIMD: each wave requests its whole first 128 keys at once
#define ATT_LAUNCH(PRE_, ONCE_)                                                                                        \
    hipLaunchKernelGGL((k_attn_mfma<DH, PRE_, ONCE_>), dim3(c.n_heads, B * row_tiles, chunks), dim3(64), 0, st,             \
                       (const bf16_t *)mod->qbuf, mod->q_plane, m, row_tiles, cache_len, geo, layer, (const bf16_t *)kv, scale, \
                       mod->attn_part, mod->attn_chunks_max, chunk_keys, mode)
    if (chunk_keys == ATT_CHUNK && chunks * items <= 1024)
        ATT_LAUNCH(4, false);
    else if (row_tiles == 1)
        ATT_LAUNCH(1, true);
    else
        ATT_LAUNCH(1, false);
#undef ATT_LAUNCH
    hipLaunchKernelGGL((k_attn_merge<DH>), dim3(B * m, c.n_heads), dim3(DH), 0, st, mod->attn_part, m, row_tiles, cache_len,
                       c.n_heads, geo.seq_pad, mod->attn_chunks_max, chunk_keys, out, mod->hd, out_plane, mod->act_mtp,
                       mode.fixed_nk);
}

// geo / kv: the cache being attended (the self-attention cache, or arch 1's cross-attention part of it);
// out / out_plane: where the merged rows go (two planes, fragment order), null = the model's shared GEMM input buffer
int32_t csd_attn_mfma_enqueue(csd_model *mod, const KvGeom &geo, const void *kv, const int32_t *cache_len, int B, int m,
                              int layer, float scale, const AttnMode &mode, hipStream_t st, bf16_t *out, size_t out_plane) {
    ProfScope ps(mod, st, CSD_PROF_ATTN);
    if (!out) {
        out = (bf16_t *)mod->act;
        out_plane = mod->act_plane;
    }
    if (mod->cfg.head_dim == 128)
        attn_launch<128>(mod, geo, kv, cache_len, B, m, layer, scale, mode, st, out, out_plane);
    else
        attn_launch<64>(mod, geo, kv, cache_len, B, m, layer, scale, mode, st, out, out_plane);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}
