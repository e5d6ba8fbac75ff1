// C-ABI entry points of libcsd: argument validation, model lifetime, and the verify step
// (review forward + softmax + accept) enqueued on the caller's stream.
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "csd_internal.h"

thread_local int32_t g_csd_last_hip_error = 0;

extern "C" const char *csd_version(void) { return "csd-mi355x 0.1 (gfx950)"; }
extern "C" int32_t csd_last_hip_error(void) { return g_csd_last_hip_error; }

static bool env_is(const char *name, const char *val) {
    const char *e = getenv(name);
    return e && strcmp(e, val) == 0;
}

// The per-call scratch of a model as one block: the residual stream, the GEMM input planes, the rotated
// queries, the split-K partial sums, the attention partial states, a probability buffer and the rotary
// table, each piece 256-byte aligned.  Returns the block's size; with base != null also the pieces.
size_t csd_scratch_carve(const csd_model *mod, char *base, ScratchPtrs *out) {
    const csd_model_cfg &c = mod->cfg;
    const size_t asz = mod->mfma ? 2 : 4, planes = mod->mfma ? 2 : 1;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = base ? base + off : nullptr;
        off += (bytes + 255) / 256 * 256;
        return p;
    };
    char *h = take(sizeof(float) * (size_t)mod->m_max * c.d_model);
    char *act = take(asz * planes * mod->act_plane);
    char *qbuf = take(asz * planes * mod->q_plane);
    char *part = take(sizeof(float) * mod->part_floats);
    char *probs = take(sizeof(float) * (size_t)mod->m_max * c.vocab);
    char *rope = take(sizeof(float2) * (size_t)mod->m_max * (c.head_dim / 2 + 1));
    char *attn_part = nullptr;
    if (mod->mfma_attn) {
        // per (sequence, head, key chunk): 16*ceil(m/16) rows x (dh accumulators + max + sum)
        const int row_tiles = (c.max_block + 15) / 16;
        const size_t per = (size_t)row_tiles * 16 * (c.head_dim + 4);
        attn_part = take(sizeof(float) * per * mod->attn_chunks_max * c.n_heads * c.max_batch);
    }
    char *x[4] = {nullptr, nullptr, nullptr, nullptr}, *ssq[2] = {nullptr, nullptr}, *cnt = nullptr;
    if (mod->chain_on) {
        for (int i = 0; i < 4; i++) x[i] = take(2 * 2 * mod->x_plane[i]);
        for (int i = 0; i < 2; i++) ssq[i] = take(sizeof(float) * (size_t)(c.d_model / 16) * 32);     // up to two row tiles
        cnt = take(sizeof(unsigned) * (size_t)c.max_batch * c.n_heads);
    }
    char *tail_rec = take(sizeof(unsigned long long) * (size_t)mod->m_max);
    char *tail_cnt = take(sizeof(unsigned) * (size_t)c.max_batch);
    char *tree_depth = take(sizeof(int32_t) * (size_t)mod->m_max);
    char *tree_anc = take(sizeof(unsigned long long) * (size_t)mod->m_max);
    char *rstd = take(sizeof(float) * (size_t)mod->m_max);
    if (out)
        *out = ScratchPtrs{(float *)h, act, qbuf, (float *)part, (float *)probs, (float2 *)rope, (float *)attn_part,
                           {x[0], x[1], x[2], x[3]}, {(float *)ssq[0], (float *)ssq[1]}, (unsigned *)cnt,
                           (unsigned long long *)tail_rec, (unsigned *)tail_cnt, (int32_t *)tree_depth,
                           (unsigned long long *)tree_anc, (float *)rstd};
    return off;
}

ScratchPtrs csd_scratch_install(csd_model *mod, const ScratchPtrs &sp) {
    const ScratchPtrs old{mod->h, mod->act, mod->qbuf, mod->part, mod->probs, mod->rope, mod->attn_part,
                          {mod->x[0], mod->x[1], mod->x[2], mod->x[3]}, {mod->ssq[0], mod->ssq[1]}, mod->attn_cnt,
                          mod->tail_rec, mod->tail_cnt, mod->tree_depth, mod->tree_anc, mod->rstd};
    mod->attn_cnt = sp.attn_cnt;
    mod->tail_rec = sp.tail_rec;
    mod->tail_cnt = sp.tail_cnt;
    mod->tree_depth = sp.tree_depth;
    mod->tree_anc = sp.tree_anc;
    mod->rstd = sp.rstd;
    for (int i = 0; i < 4; i++) mod->x[i] = sp.x[i];
    for (int i = 0; i < 2; i++) mod->ssq[i] = sp.ssq[i];
    mod->h = sp.h;
    mod->act = sp.act;
    mod->qbuf = sp.qbuf;
    mod->part = sp.part;
    mod->probs = sp.probs;
    mod->rope = sp.rope;
    mod->attn_part = sp.attn_part;
    return old;
}

__global__ void k_fill_u32(unsigned *__restrict__ p, unsigned v, int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = v;
}

// Scratch for csd_verify_accept_static: one copy per device, held until the process ends.  In host code the
// array's name is only a handle for the symbol look-up; the device address comes from hipGetSymbolAddress,
// once per device, and is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[CSD_STATIC_SCRATCH_BYTES];
static char *g_static_base[64];
static std::mutex g_static_mu;

static int32_t static_scratch_base(char **out) {
    int dev = -1;
    CSD_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return CSD_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_base[dev]) {
        void *p = nullptr;
        CSD_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return CSD_EHIP;
        g_static_base[dev] = (char *)p;
    }
    *out = g_static_base[dev];
    return CSD_OK;
}

static int32_t create_impl(csd_model *mod, const void *const *weights, hipStream_t st) {
    const csd_model_cfg &c = mod->cfg;
    mod->hd = c.n_heads * c.head_dim;
    mod->seq_pad = (c.max_seq + 63) / 64 * 64;
    mod->enc_pad = c.arch == 1 ? (c.enc_len + 63) / 64 * 64 : 0;
    mod->m_max = c.max_batch * c.max_block;
    const int d = c.d_model, F = c.d_ffn, hd = mod->hd, V = c.vocab;
    // The MFMA path needs whole 16-feature tiles and 32-wide k-steps everywhere.
    const bool tiles_ok = d % 32 == 0 && hd % 32 == 0 && F % 32 == 0 && V % 16 == 0 && c.head_dim % 16 == 0;
    mod->mfma = c.dtype == CSD_DTYPE_BF16 && tiles_ok && !env_is("CSD_GEMM", "generic");
    mod->kperm = mod->mfma && c.arch == 0;     // rotary pair order only where there is a rotary embedding
    mod->mfma_attn = mod->mfma && (c.head_dim == 64 || c.head_dim == 128) && !env_is("CSD_ATTN", "generic");
    const int keys_pad = mod->seq_pad > mod->enc_pad ? mod->seq_pad : mod->enc_pad;
    if (!mod->mfma_attn && sizeof(float) * (size_t)(c.head_dim + keys_pad) > 64 * 1024) return CSD_ESHAPE;
    {
        // the GEMM kernels address a matrix through one buffer descriptor with 32-bit offsets
        const size_t esz = c.dtype == CSD_DTYPE_BF16 ? 2 : 4;
        const size_t mats[5] = {(size_t)d * 3 * hd, (size_t)hd * d, (size_t)d * 2 * F, (size_t)F * d, (size_t)d * V};
        for (size_t n : mats)
            if (n * esz >= ((size_t)1 << 31)) return CSD_ESHAPE;
    }
    int32_t rc;
    if ((rc = csd_pack_weights(mod, weights, st)) != CSD_OK) return rc;
    if (mod->mfma && (rc = csd_gemm_setup()) != CSD_OK) return rc;

    const int m_pad = (mod->m_max + 15) / 16 * 16;
    int wmax = d > F ? d : F;
    if (hd > wmax) wmax = hd;
    int nmax = 3 * hd;
    if (2 * F > nmax) nmax = 2 * F;
    if (V > nmax) nmax = V;
    if (d > nmax) nmax = d;
    mod->act_plane = (size_t)m_pad * wmax;
    mod->act_mtp = mod->mfma ? m_pad / 16 : 0;
    mod->q_plane = (size_t)m_pad * hd;
    mod->part_floats = (size_t)mod->s_max * mod->m_max * nmax;
    if (mod->mfma_attn) mod->attn_chunks_max = (keys_pad + 127) / 128;
    // blocks of up to 32 rows of a bf16 model (either architecture) take the forward of csd_chain.hip (CSD_PATH=multikernel: never)
    mod->chain_on = mod->mfma && mod->mfma_attn && (mod->kperm || c.arch == 1) && !env_is("CSD_PATH", "multikernel");
    if (mod->chain_on) {
        const int widths[4] = {d, hd, d, F};
        for (int i = 0; i < 4; i++) mod->x_plane[i] = (size_t)m_pad * widths[i];
        if ((rc = csd_chain_setup()) != CSD_OK) return rc;
    }
    // the per-call scratch is one block, carved the same way wherever it lives
    void *p;
    CSD_HIP(hipMalloc(&p, csd_scratch_carve(mod, nullptr, nullptr)));
    mod->allocs.push_back(p);
    ScratchPtrs sp;
    csd_scratch_carve(mod, (char *)p, &sp);
    csd_scratch_install(mod, sp);
    if (mod->attn_cnt) {     // arrival counters start at zero; every launch leaves them there
        hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(256), 0, st, mod->attn_cnt, 0u, c.max_batch * c.n_heads);
        CSD_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(256), 0, st, mod->tail_cnt, 0u, c.max_batch);
    CSD_LAUNCH_CHECK();
    char *static_base;
    if ((rc = static_scratch_base(&static_base)) != CSD_OK) return rc;   // looked up once per device, here
    CSD_HIP(hipMalloc(&p, sizeof(int32_t) * (size_t)mod->m_max));
    mod->allocs.push_back(p);
    mod->review_block = (int32_t *)p;
    mod->ev.resize(8192);
    for (auto &e : mod->ev) CSD_HIP(hipEventCreate(&e));
    return CSD_OK;
}

extern "C" int32_t csd_model_create(const csd_model_cfg *cfg, const void *const *weight_ptrs, int32_t n_weights,
                                    void *stream, csd_model **out) {
    if (!cfg || !weight_ptrs || !out) return CSD_ENULL;
    *out = nullptr;
    if (cfg->arch != 0 && cfg->arch != 1) return CSD_EUNSUPPORTED;
    if ((cfg->arch == 0 && cfg->enc_len != 0) || (cfg->arch == 1 && cfg->enc_len < 1)) return CSD_EINVAL;
    if (cfg->dtype != CSD_DTYPE_FP32 && cfg->dtype != CSD_DTYPE_BF16) return CSD_EINVAL;
    if (cfg->n_layers < 1 || cfg->d_model < 1 || cfg->n_heads < 1 || cfg->head_dim < 2 || cfg->head_dim % 2 ||
        cfg->d_ffn < 1 || cfg->vocab < 1 || cfg->max_batch < 1 || cfg->max_seq < 1 || cfg->max_block < 1)
        return CSD_EINVAL;
    if (!(cfg->rms_eps > 0.f) || (cfg->arch == 0 && !(cfg->rope_theta > 0.f))) return CSD_EINVAL;
    if (cfg->max_block > cfg->max_seq) return CSD_ESHAPE;
    if ((long long)cfg->max_batch * cfg->max_block > 4096) return CSD_ESHAPE;
    if (n_weights != (cfg->arch == 0 ? 3 + 9 * cfg->n_layers : 4 + 14 * cfg->n_layers)) return CSD_EINVAL;
    for (int i = 0; i < n_weights; i++)
        if (!weight_ptrs[i]) return CSD_ENULL;
    csd_model *mod = new (std::nothrow) csd_model();
    if (!mod) return CSD_EHIP;
    mod->cfg = *cfg;
    const int32_t rc = create_impl(mod, weight_ptrs, (hipStream_t)stream);
    if (rc != CSD_OK) {
        csd_model_destroy(mod);
        return rc;
    }
    *out = mod;
    return CSD_OK;
}

extern "C" int32_t csd_model_destroy(csd_model *mod) {
    if (!mod) return CSD_ENULL;
    for (void *p : mod->allocs) (void)hipFree(p);
    for (auto &e : mod->ev)
        if (e) (void)hipEventDestroy(e);
    delete mod;
    return CSD_OK;
}

static int32_t check_block(const csd_model *mod, const void *kv, const int32_t *tokens, const int32_t *cache_len,
                           int32_t B, int32_t m) {
    if (!mod || !kv || !tokens || !cache_len) return CSD_ENULL;
    if (B < 1 || m < 1) return CSD_EINVAL;
    if (B > mod->cfg.max_batch || m > mod->cfg.max_block) return CSD_ESHAPE;
    return CSD_OK;
}

extern "C" int32_t csd_verify_block(csd_model *mod, void *kv, const int32_t *tokens, const int32_t *cache_len,
                                    int32_t B, int32_t m, float temperature, float *logits, float *probs,
                                    void *stream) {
    int32_t rc = check_block(mod, kv, tokens, cache_len, B, m);
    if (rc != CSD_OK) return rc;
    if (!logits) return CSD_ENULL;
    if (probs && !(temperature > 0.f)) return CSD_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    if ((rc = csd_forward_enqueue(mod, kv, tokens, cache_len, B, m, logits, st)) != CSD_OK) return rc;
    if (probs) {
        ProfScope ps(mod, st, CSD_PROF_OTHER);
        if ((rc = csd_softmax_enqueue(logits, probs, (int64_t)B * m, mod->cfg.vocab, temperature, st)) != CSD_OK) return rc;
    }
    return CSD_OK;
}

// Depth and ancestor mask of every row of a tree block.  parent[b][i] < i names the row that row i continues
// (row 0 has none); a value outside [0, i) is read as 0, so the walk up always ends at row 0.
__global__ void k_tree_prepare(const int32_t *__restrict__ parent, int m, int32_t *__restrict__ depth,
                               unsigned long long *__restrict__ anc) {
    const int b = blockIdx.x, i = threadIdx.x;
    if (i >= m) return;
    const int32_t *par = parent + (size_t)b * m;
    unsigned long long mask = 1ull << i;
    int d = 0, r = i;
    while (r > 0) {
        int pr = par[r];
        if (pr < 0 || pr >= r) pr = 0;
        mask |= 1ull << pr;
        d++;
        r = pr;
    }
    depth[b * m + i] = d;
    anc[b * m + i] = mask;
}

// After a tree review: the K/V of the kept rows path[b][0 .. n) move to cache rows cache_len + 1 .., where a plain
// block would have stored them.  A thread owns one feature of one (layer, sequence, head) and moves it row by row, in
// order (path is increasing and path[j] >= j + 1, so nothing still needed is overwritten); a path that is not of
// that form is cut at the first offending entry.
template <typename TC>
__global__ void k_tree_commit(TC *__restrict__ kv, KvGeom geo, const int32_t *__restrict__ cache_len,
                              const int32_t *__restrict__ path, const int32_t *__restrict__ n_accepted, int m) {
    const int l = blockIdx.x, b = blockIdx.y, hh = blockIdx.z, x = threadIdx.x;
    const int t = cache_len[b];
    int n = n_accepted[b];
    n = n < 0 ? 0 : (n > m - 1 ? m - 1 : n);
    TC *kc = kv + kv_k_off(geo, l, b, hh);
    TC *vc = kv + kv_v_off(geo, l, b, hh);
    int prev = 0;
    for (int j = 0; j < n; j++) {
        const int src = path[(size_t)b * m + j];
        if (src <= prev || src < j + 1 || src >= m || t < 0 || t + src >= geo.seq_pad) break;
        prev = src;
        if (src == j + 1) continue;                          // already where it belongs
        const int from = t + src, to = t + 1 + j;
        kc[(size_t)to * geo.dh + x] = kc[(size_t)from * geo.dh + x];
        vc[kv_v_idx(geo, x, to)] = vc[kv_v_idx(geo, x, from)];
    }
}

extern "C" int32_t csd_verify_tree(csd_model *mod, void *kv, const int32_t *tokens, const int32_t *parent,
                                   const int32_t *cache_len, int32_t B, int32_t m, float temperature, float *logits,
                                   float *probs, void *stream) {
    int32_t rc = check_block(mod, kv, tokens, cache_len, B, m);
    if (rc != CSD_OK) return rc;
    if (!logits || !parent) return CSD_ENULL;
    if (mod->cfg.arch != 0) return CSD_EUNSUPPORTED;
    if (m > 64) return CSD_ESHAPE;                           // a row's ancestors are one 64-bit mask
    if (probs && !(temperature > 0.f)) return CSD_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(k_tree_prepare, dim3(B), dim3(64), 0, st, parent, m, mod->tree_depth, mod->tree_anc);
    CSD_LAUNCH_CHECK();
    mod->tree_call = true;                                   // the kernels take the two arrays as arguments at enqueue time
    rc = csd_forward_enqueue(mod, kv, tokens, cache_len, B, m, logits, st);
    mod->tree_call = false;
    if (rc != CSD_OK) return rc;
    if (probs) {
        ProfScope ps(mod, st, CSD_PROF_OTHER);
        if ((rc = csd_softmax_enqueue(logits, probs, (int64_t)B * m, mod->cfg.vocab, temperature, st)) != CSD_OK) return rc;
    }
    return CSD_OK;
}

extern "C" int32_t csd_tree_commit(const csd_model *mod, void *kv, const int32_t *cache_len, const int32_t *path,
                                   const int32_t *n_accepted, int32_t B, int32_t m, void *stream) {
    if (!mod || !kv || !cache_len || !path || !n_accepted) return CSD_ENULL;
    if (B < 1 || m < 1) return CSD_EINVAL;
    if (B > mod->cfg.max_batch || m > mod->cfg.max_block || m > 64) return CSD_ESHAPE;
    if (mod->cfg.arch != 0) return CSD_EUNSUPPORTED;
    const csd_model_cfg &c = mod->cfg;
    const KvGeom geo{c.max_batch, c.n_heads, c.head_dim, mod->seq_pad, c.n_layers, mod->kperm ? 1 : 0};
    const dim3 grid(c.n_layers, B, c.n_heads);
    if (c.dtype == CSD_DTYPE_BF16)
        hipLaunchKernelGGL((k_tree_commit<bf16_t>), grid, dim3(c.head_dim), 0, (hipStream_t)stream, (bf16_t *)kv, geo, cache_len,
                           path, n_accepted, m);
    else
        hipLaunchKernelGGL((k_tree_commit<float>), grid, dim3(c.head_dim), 0, (hipStream_t)stream, (float *)kv, geo, cache_len,
                           path, n_accepted, m);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

extern "C" int32_t csd_verify_accept(csd_model *mod, void *kv, const int32_t *tokens, const int32_t *cache_len,
                                     int32_t B, int32_t m, float temperature, const float *q, const uint8_t *q_onehot,
                                     const float *u_acc, const float *u_samp, float lenience, int32_t mode,
                                     float *logits, float *probs, int32_t *n_accepted, int32_t *next_token,
                                     void *stream) {
    int32_t rc = check_block(mod, kv, tokens, cache_len, B, m);
    if (rc != CSD_OK) return rc;
    if (!n_accepted || !next_token) return CSD_ENULL;
    if (mode != CSD_MODE_SAMPLE && mode != CSD_MODE_GREEDY) return CSD_EINVAL;
    if (!(lenience >= 1.0f) || lenience > 256.0f) return CSD_EINVAL;
    const bool need_probs = mode == CSD_MODE_SAMPLE || lenience > 1.0f;
    if (need_probs && !(temperature > 0.f)) return CSD_EINVAL;
    if (mode == CSD_MODE_SAMPLE && (!u_samp || (m > 1 && !u_acc))) return CSD_ENULL;
    hipStream_t st = (hipStream_t)stream;
    const int V = mod->cfg.vocab;
    // logits of this call live in the model's scratch when the caller does not ask for them
    float *lg = logits ? logits : mod->probs;   // softmax may then run in place: each thread rewrites what it read
    if ((rc = csd_forward_enqueue(mod, kv, tokens, cache_len, B, m, lg, st)) != CSD_OK) return rc;
    if (csd_review_rows_fits(lg, probs, q, V)) {
        // one launch: every row normalised (if anything needs probabilities), tested and its replacement drawn at
        // once; probabilities are written only for a caller that asks for them
        ProfScope ps(mod, st, CSD_PROF_OTHER);
        return csd_review_rows_enqueue(lg, probs, mod->tail_rec, mod->tail_cnt, temperature, q, q_onehot, tokens + 1, m, u_acc,
                                       u_samp, B, m - 1, V, lenience, mode, n_accepted, next_token, st);
    }
    const float *p = lg;
    if (need_probs || probs) {
        float *pr = probs ? probs : mod->probs;
        ProfScope ps(mod, st, CSD_PROF_OTHER);
        if ((rc = csd_softmax_enqueue(lg, pr, (int64_t)B * m, V, temperature > 0.f ? temperature : 1.0f, st)) != CSD_OK)
            return rc;
        if (need_probs) p = pr;
    }
    ProfScope ps(mod, st, CSD_PROF_OTHER);
    return csd_accept_enqueue(p, q, q_onehot, tokens + 1, m, u_acc, u_samp, B, m - 1, V, lenience, mode, n_accepted,
                              next_token, st);
}

extern "C" int32_t csd_verify_accept_static(csd_model *mod, void *kv, const int32_t *tokens, const int32_t *cache_len,
                                            int32_t B, int32_t m, float temperature, const float *q,
                                            const uint8_t *q_onehot, const float *u_acc, const float *u_samp,
                                            float lenience, int32_t mode, float *logits, float *probs,
                                            int32_t *n_accepted, int32_t *next_token, void *stream) {
    if (!mod) return CSD_ENULL;
    if (csd_scratch_carve(mod, nullptr, nullptr) > CSD_STATIC_SCRATCH_BYTES) return CSD_ESHAPE;
    char *base;
    int32_t rc = static_scratch_base(&base);
    if (rc != CSD_OK) return rc;
    ScratchPtrs sp;
    csd_scratch_carve(mod, base, &sp);
    // the kernels take the scratch pieces as arguments at enqueue time, so the model's own pieces are back in
    // place as soon as the enqueue returns
    const ScratchPtrs own = csd_scratch_install(mod, sp);
    if (sp.attn_cnt) {
        // the array keeps whatever the last call on this GPU left (another model lays it out differently): the
        // attention kernel's arrival counters must start at zero.  A fill kernel, not a memset: the call may be
        // under graph capture.
        hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(256), 0, (hipStream_t)stream, sp.attn_cnt, 0u,
                           mod->cfg.max_batch * mod->cfg.n_heads);
    }
    hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(256), 0, (hipStream_t)stream, sp.tail_cnt, 0u, mod->cfg.max_batch);
    rc = csd_verify_accept(mod, kv, tokens, cache_len, B, m, temperature, q, q_onehot, u_acc, u_samp, lenience, mode,
                           logits, probs, n_accepted, next_token, stream);
    csd_scratch_install(mod, own);
    return rc;
}

extern "C" int32_t csd_debug_set_trace(csd_model *mod, float *trace) {
    if (!mod) return CSD_ENULL;
    mod->trace = trace;
    return CSD_OK;
}

extern "C" int32_t csd_debug_path(const csd_model *mod, int32_t B, int32_t m) {
    if (!mod) return CSD_ENULL;
    return csd_chain_eligible(mod, B, m) ? 1 : 0;
}

extern "C" int32_t csd_debug_gemm_plan(int32_t N, int32_t K, int32_t rows, int32_t max_splits, int32_t *ct, int32_t *S) {
    if (max_splits < 1) return CSD_EINVAL;
    return csd_rs_plan_host(N, K, rows, (size_t)max_splits * (size_t)rows * (size_t)N, ct, S);
}

__global__ __launch_bounds__(256) void k_copy_calib(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

extern "C" int32_t csd_debug_copy(void *dst, const void *src, size_t bytes, void *stream) {
    if (!dst || !src) return CSD_ENULL;
    if (bytes % 16 || ((uintptr_t)dst | (uintptr_t)src) % 16) return CSD_EINVAL;
    if (bytes == 0) return CSD_OK;
    hipLaunchKernelGGL(k_copy_calib, dim3(256 * 8), dim3(256), 0, (hipStream_t)stream, (u32x4 *)dst, (const u32x4 *)src,
                       bytes / 16);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

__global__ __launch_bounds__(256) void k_read_calib(const u32x4 *__restrict__ src, size_t n, uint32_t *__restrict__ sink) {
    u32x4 acc = u32x4{0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        acc ^= __builtin_nontemporal_load(src + i);
    const uint32_t v = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    if (v == 0x9E3779B9u || threadIdx.x == 0) sink[blockIdx.x] = v;      // keeps every lane's loads
}

extern "C" int32_t csd_debug_read(const void *src, size_t bytes, uint32_t *sink, void *stream) {
    if (!src || !sink) return CSD_ENULL;
    if (bytes % 16 || (uintptr_t)src % 16) return CSD_EINVAL;
    if (bytes == 0) return CSD_OK;
    hipLaunchKernelGGL(k_read_calib, dim3(2048), dim3(256), 0, (hipStream_t)stream, (const u32x4 *)src, bytes / 16, sink);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

__global__ __launch_bounds__(256) void k_mfma_calib(long long iters, uint32_t *__restrict__ sink) {
    const uint32_t seed = 0x3F803F80u + (threadIdx.x & 7u);              // small bf16 values
    const bf16x8 a = __builtin_bit_cast(bf16x8, u32x4{seed, seed, seed, seed});
    const bf16x8 b = __builtin_bit_cast(bf16x8, u32x4{0x3C003C00u, 0x3C003C00u, 0x3C003C00u, 0x3C003C00u});
    f32x4 acc[8];
#pragma unroll
    for (int j = 0; j < 8; j++) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (long long i = 0; i < iters; i++) {
#pragma unroll
        for (int j = 0; j < 8; j++) acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[j], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < 8; j++) t += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
    if (t == -1.0f || threadIdx.x == 0) sink[blockIdx.x] = __float_as_uint(t);
}

extern "C" int32_t csd_debug_mfma(int64_t iters, uint32_t *sink, void *stream) {
    if (!sink) return CSD_ENULL;
    if (iters < 0 || iters > (1ll << 24)) return CSD_EINVAL;
    if (iters == 0) return CSD_OK;
    hipLaunchKernelGGL(k_mfma_calib, dim3(1024), dim3(256), 0, (hipStream_t)stream, (long long)iters, sink);
    CSD_LAUNCH_CHECK();
    return CSD_OK;
}

extern "C" int32_t csd_prof_enable(csd_model *mod, int32_t on) {
    if (!mod) return CSD_ENULL;
    mod->prof = on != 0;
    return CSD_OK;
}

extern "C" int32_t csd_prof_read(csd_model *mod, int32_t cls, double *ms, int64_t *launches, int32_t reset) {
    if (!mod || !ms || !launches) return CSD_ENULL;
    if (cls < 0 || cls >= CSD_PROF_CLASSES) return CSD_EINVAL;
    // fold finished event pairs into the per-class totals (the caller has synchronised the stream)
    for (size_t i = 0; i + 1 < mod->ev_used; i += 2) {
        float t = 0.f;
        CSD_HIP(hipEventElapsedTime(&t, mod->ev[i], mod->ev[i + 1]));
        const int k = mod->ev_class[i / 2];
        mod->prof_ms[k] += t;
        mod->prof_n[k] += 1;
    }
    mod->ev_used = 0;
    mod->ev_class.clear();
    *ms = mod->prof_ms[cls];
    *launches = mod->prof_n[cls];
    if (reset)
        for (int k = 0; k < CSD_PROF_CLASSES; k++) {
            mod->prof_ms[k] = 0;
            mod->prof_n[k] = 0;
        }
    return CSD_OK;
}
