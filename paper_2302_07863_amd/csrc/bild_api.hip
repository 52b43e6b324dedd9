// C ABI of the BiLD library: model upload, per-request state, and the launch
// sequences of the decoder passes.  All numerical work is in kernels.hip; this
// file owns memory and ordering only.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <array>
#include <cmath>
#include <cstdlib>
#include <map>
#include <cstdio>
#include <chrono>
#include <cstring>
#include <new>
#include <vector>

#include "bild_state.h"

using namespace bild;

namespace bild {
int dev_alloc(std::vector<void*>& keep, void** p, size_t bytes) {
    void* d = nullptr;
    if (bytes == 0) bytes = 16;
    if (hipMalloc(&d, bytes) != hipSuccess) return BILD_ENOMEM;
    keep.push_back(d);
    *p = d;
    return BILD_OK;
}
}  // namespace bild

namespace {

// ---------------------------------------------------------------- helpers

bool config_ok(const bild_model_config& c) {
    if (c.n_dec_layers < 1 || c.n_enc_layers < 0) return false;
    if (c.d_model < 32 || c.d_model % 32 || c.d_ff < 32 || c.d_ff % 32) return false;
    if (c.n_heads < 1 || c.d_head < 8 || c.d_head > 128 || c.d_head % 8) return false;
    if ((c.n_heads * c.d_head) % 32) return false;
    if (c.act < 0 || c.act > 2 || c.pos < 0 || c.pos > 2 || c.dtype < 0 || c.dtype > 1) return false;
    if (c.vocab < 1 || c.bos < 0 || c.bos >= c.vocab) return false;
    if (c.n_enc_layers > 0 && !c.cross_attn) return false;
    if (!(c.norm_eps >= 0.f) || !(c.rope_base > 0.f)) return false;
    if (c.tie_shift < 0) return false;
    if (c.pos == BILD_POS_RELATIVE && (c.rel_max_dist < 1 || c.rel_max_dist > 4096)) return false;
    return true;
}

int upload_vec(bild_model* m, const float* src, int n, const float** out) {
    void* d;
    int rc = dev_alloc(m->allocs, &d, (size_t)n * 4);
    if (rc) return rc;
    if (hipMemcpy(d, src, (size_t)n * 4, hipMemcpyHostToDevice) != hipSuccess) return BILD_EHIP;
    m->device_bytes += (size_t)n * 4;
    *out = (const float*)d;
    return BILD_OK;
}

int upload_tiled(bild_model* m, std::vector<char>& staging, int n, int k, TMat* out) {
    const int kt = m->cfg.dtype == BILD_DT_BF16 ? 32 : 16;
    const size_t bytes = tiled_bytes(n, k, m->cfg.dtype);
    void* d;
    int rc = dev_alloc(m->allocs, &d, bytes);
    if (rc) return rc;
    if (hipMemcpy(d, staging.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) return BILD_EHIP;
    m->device_bytes += bytes;
    out->w = d;
    out->n = n;
    out->k = k;
    out->tn = (n + 15) / 16;
    out->tk = k / kt;
    return BILD_OK;
}

int upload_matrix(bild_model* m, const float* src, bool k_by_n, int n, int k, TMat* out) {
    std::vector<char> st(tiled_bytes(n, k, m->cfg.dtype));
    tile_matrix(src, k_by_n, n, k, m->cfg.dtype, st.data());
    return upload_tiled(m, st, n, k, out);
}

int upload_concat(bild_model* m, std::initializer_list<const float*> srcs, int n_each, int k, TMat* out) {
    std::vector<const float*> ps(srcs);
    std::vector<int> ns(ps.size(), n_each);
    const int n = n_each * (int)ps.size();
    std::vector<char> st(tiled_bytes(n, k, m->cfg.dtype));
    tile_concat(ps.data(), ns.data(), (int)ps.size(), k, m->cfg.dtype, st.data());
    return upload_tiled(m, st, n, k, out);
}

int upload_ffn_in(bild_model* m, const float* w_in, const float* w_up, TMat* out) {
    const int d = m->cfg.d_model, f = m->cfg.d_ff;
    if (!m->gated()) return upload_matrix(m, w_in, true, f, d, out);
    std::vector<char> st(tiled_bytes(2 * f, d, m->cfg.dtype));
    tile_gated_pair(w_in, w_up, f, d, m->cfg.dtype, st.data());
    return upload_tiled(m, st, 2 * f, d, out);
}

}  // namespace

// ======================================================================= models
extern "C" int bild_model_num_tensors(const bild_model_config* c) {
    if (!c || !config_ok(*c)) return BILD_EINVAL;
    const int gated = c->act != BILD_ACT_RELU;
    int n = 1 + (c->tied_head ? 0 : 1) + (c->n_enc_layers > 0 ? 1 : 0) + 1;
    if (c->pos == BILD_POS_RELATIVE) n += (c->n_enc_layers > 0 ? 1 : 0) + 1;
    n += c->n_enc_layers * (8 + gated);
    n += c->n_dec_layers * (8 + gated + (c->cross_attn ? 5 : 0));
    return n;
}

extern "C" int bild_model_destroy(bild_model* m) {
    if (!m) return BILD_EINVAL;
    for (void* p : m->allocs) (void)hipFree(p);
    delete m;
    return BILD_OK;
}

extern "C" int bild_model_create(const bild_model_config* cfg, const float* const* t, int n_tensors,
                                 bild_model** out) {
    if (!cfg || !t || !out) return BILD_EINVAL;
    if (!config_ok(*cfg)) return BILD_EINVAL;
    if (n_tensors != bild_model_num_tensors(cfg)) return BILD_EINVAL;
    for (int i = 0; i < n_tensors; ++i)
        if (!t[i]) return BILD_EINVAL;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return BILD_EHIP;
    bild_model* m = new (std::nothrow) bild_model();
    if (!m) return BILD_ENOMEM;
    m->cfg = *cfg;
    const int d = cfg->d_model, I = m->inner(), F = cfg->d_ff, V = cfg->vocab;
    int i = 0, rc = BILD_OK;
#define UP(call)                         \
    do {                                 \
        rc = (call);                     \
        if (rc) {                        \
            bild_model_destroy(m);       \
            return rc;                   \
        }                                \
    } while (0)
    UP(upload_matrix(m, t[i++], false, V, d, &m->emb));
    if (cfg->tied_head)
        m->head = m->emb;
    else
        UP(upload_matrix(m, t[i++], false, V, d, &m->head));
    if (cfg->n_enc_layers > 0) UP(upload_vec(m, t[i++], d, &m->enc_final));
    UP(upload_vec(m, t[i++], d, &m->dec_final));
    if (cfg->pos == BILD_POS_RELATIVE) {
        const int nrel = cfg->n_heads * (2 * cfg->rel_max_dist + 1);
        if (cfg->n_enc_layers > 0) UP(upload_vec(m, t[i++], nrel, &m->enc_rel));
        UP(upload_vec(m, t[i++], nrel, &m->dec_rel));
    }
    m->enc.resize(cfg->n_enc_layers);
    for (auto& L : m->enc) {
        UP(upload_vec(m, t[i], d, &L.ln1));
        UP(upload_concat(m, {t[i + 1], t[i + 2], t[i + 3]}, I, d, &L.wqkv));
        UP(upload_matrix(m, t[i + 4], true, d, I, &L.wo));
        UP(upload_vec(m, t[i + 5], d, &L.ln2));
        i += 6;
        UP(upload_ffn_in(m, t[i], m->gated() ? t[i + 1] : nullptr, &L.win));
        i += m->gated() ? 2 : 1;
        UP(upload_matrix(m, t[i++], true, d, F, &L.wout));
    }
    m->dec.resize(cfg->n_dec_layers);
    for (auto& L : m->dec) {
        UP(upload_vec(m, t[i], d, &L.ln1));
        UP(upload_concat(m, {t[i + 1], t[i + 2], t[i + 3]}, I, d, &L.wqkv));
        UP(upload_matrix(m, t[i + 4], true, d, I, &L.wo));
        i += 5;
        if (cfg->cross_attn) {
            UP(upload_vec(m, t[i], d, &L.lnc));
            UP(upload_matrix(m, t[i + 1], true, I, d, &L.cwq));
            UP(upload_concat(m, {t[i + 2], t[i + 3]}, I, d, &L.cwkv));
            UP(upload_matrix(m, t[i + 4], true, d, I, &L.cwo));
            i += 5;
        }
        UP(upload_vec(m, t[i++], d, &L.ln2));
        UP(upload_ffn_in(m, t[i], m->gated() ? t[i + 1] : nullptr, &L.win));
        i += m->gated() ? 2 : 1;
        UP(upload_matrix(m, t[i++], true, d, F, &L.wout));
    }
#undef UP
    *out = m;
    return BILD_OK;
}

extern "C" int bild_pair_create(bild_model* s, bild_model* l, bild_pair** out) {
    if (!s || !l || !out) return BILD_EINVAL;
    if (s->cfg.vocab != l->cfg.vocab) return BILD_EINVAL;
    if (s->cfg.cross_attn != l->cfg.cross_attn) return BILD_EINVAL;
    if (s->cfg.bos != l->cfg.bos) return BILD_EINVAL;
    const bool dec_only = !l->cfg.cross_attn;
    bool borrows = false;
    if (!dec_only) {
        if (l->cfg.n_enc_layers < 1) return BILD_EINVAL;
        if (s->cfg.n_enc_layers == 0) {
            if (s->cfg.d_model != l->cfg.d_model) return BILD_EINVAL;
            borrows = true;
        }
    }
    bild_pair* p = new (std::nothrow) bild_pair();
    if (!p) return BILD_ENOMEM;
    p->m[0] = s;
    p->m[1] = l;
    p->decoder_only = dec_only;
    p->small_borrows_encoder = borrows;
    *out = p;
    return BILD_OK;
}

extern "C" int bild_pair_create_early_exit(bild_model* l, int k, float small_logit_scale, bild_pair** out) {
    if (!l || !out) return BILD_EINVAL;
    if (k < 1 || k >= l->cfg.n_dec_layers || !(small_logit_scale > 0.f)) return BILD_EINVAL;
    if (l->cfg.cross_attn && l->cfg.n_enc_layers < 1) return BILD_EINVAL;
    bild_model* v = new (std::nothrow) bild_model();
    bild_pair* p = new (std::nothrow) bild_pair();
    if (!v || !p) {
        delete v;
        delete p;
        return BILD_ENOMEM;
    }
    v->cfg = l->cfg;
    v->cfg.n_dec_layers = k;
    v->cfg.n_enc_layers = 0;  // it attends to the large model's encoder output
    v->cfg.logit_scale = small_logit_scale;
    v->emb = l->emb;
    v->head = l->head;
    v->dec_final = l->dec_final;
    v->dec_rel = l->dec_rel;
    v->dec.assign(l->dec.begin(), l->dec.begin() + k);
    p->m[0] = v;
    p->m[1] = l;
    p->decoder_only = !l->cfg.cross_attn;
    p->small_borrows_encoder = l->cfg.cross_attn != 0;
    p->trunk_layers = k;
    p->view = v;
    *out = p;
    return BILD_OK;
}

extern "C" int bild_pair_destroy(bild_pair* p) {
    if (!p) return BILD_EINVAL;
    delete p->view;  // a view owns no device memory
    delete p;
    return BILD_OK;
}

// ======================================================================= state
extern "C" int bild_state_destroy(bild_state* s) {
    if (!s) return BILD_EINVAL;
    if (s->stream) (void)hipStreamSynchronize(s->stream);
    for (void* p : s->allocs) (void)hipFree(p);
    for (void* p : s->host_allocs) (void)hipHostFree(p);
    for (hipEvent_t e : s->prof_ev) (void)hipEventDestroy(e);
    for (auto& kv : s->graphs) (void)hipGraphExecDestroy(kv.second);
    if (s->own_stream && s->stream) (void)hipStreamDestroy(s->stream);
    delete s;
    return BILD_OK;
}

extern "C" int bild_state_create(const bild_pair* p, int max_src, int max_len, int n_max, void* hip_stream,
                                 bild_state** out) {
    if (!p || !out) return BILD_EINVAL;
    if (max_src < 1 || max_len < 2 || n_max < 0 || n_max > kMaxRows - 1) return BILD_EINVAL;
    if (p->decoder_only && max_len < max_src + 1) return BILD_EINVAL;
    bild_state* s = new (std::nothrow) bild_state();
    if (!s) return BILD_ENOMEM;
    s->pair = p;
    s->max_src = max_src;
    s->max_len = max_len;
    s->n_max = n_max;
    s->cap_len = (max_len + 31) / 32 * 32;
    s->cap_src = (max_src + 31) / 32 * 32;
    if (kernels_init() != hipSuccess) {
        delete s;
        return BILD_EHIP;
    }
    int rc = BILD_OK;
#define AL(ptr, bytes)                                            \
    do {                                                          \
        rc = dev_alloc(s->allocs, (void**)&(ptr), (bytes));       \
        if (rc) {                                                 \
            bild_state_destroy(s);                                \
            return rc;                                            \
        }                                                         \
    } while (0)
    if (hip_stream) {
        s->stream = (hipStream_t)hip_stream;
    } else {
        if (hipStreamCreate(&s->stream) != hipSuccess) {
            delete s;
            return BILD_EHIP;
        }
        s->own_stream = true;
    }
    AL(s->ctl, sizeof(Ctl));
    AL(s->y, sizeof(int) * (size_t)(max_len + 1));
    AL(s->src, sizeof(int) * (size_t)max_src);
    void* h = nullptr;
    if (hipHostMalloc(&h, sizeof(Ctl) + 64, hipHostMallocMapped) != hipSuccess) {
        bild_state_destroy(s);
        return BILD_ENOMEM;
    }
    s->host_allocs.push_back(h);
    s->hctl = (Ctl*)h;
    s->halpha = (float*)((char*)h + sizeof(Ctl));
    void* hd = nullptr;
    if (hipHostGetDevicePointer(&hd, h, 0) != hipSuccess) {
        bild_state_destroy(s);
        return BILD_EHIP;
    }
    s->hctl_dev = (Ctl*)hd;
    {
        const char* ng = std::getenv("BILD_NO_GRAPH");
        s->use_graphs = !(ng && ng[0] == '1');
        if (const char* pm = std::getenv("BILD_PRE_MIN_ROWS")) s->pre_min_rows = std::atoi(pm);  // experiments; > 32 turns the planes off
        if (const char* fa = std::getenv("BILD_FUSE_ATTN")) s->fuse_attn = fa[0] != '0';      // experiments / tests
        if (const char* fk = std::getenv("BILD_FUSE_MAX_KV")) s->fuse_max_kv = std::atoi(fk);
        if (const char* dw = std::getenv("BILD_DRAW_ONE_WG")) s->draw_spread = dw[0] == '0';
        if (const char* fe = std::getenv("BILD_FUSE_EMBED")) s->fuse_embed = std::atoi(fe) != 0;  // tests and measurements
        if (const char* kd = std::getenv("BILD_KSPLIT_MAX_D")) s->ksplit_max_d = std::atoi(kd);
        if (const char* km = std::getenv("BILD_KSPLIT_MIN_F")) s->ksplit_min_f = std::atoi(km);  // tests: small widths; 0 turns the split off
    }
    for (int w = 0; w < 2; ++w) {
        ModelState& M = s->ms[w];
        const bild_model* m = p->m[w];
        M.m = m;
        const size_t I = m->inner(), d = m->cfg.d_model, F = m->cfg.d_ff, L = m->cfg.n_dec_layers;
        const size_t esz = m->esz();
        // every K/V buffer starts zeroed: rows past the valid length must hold finite values
#define ALZ(ptr, bytes)                                                              \
    do {                                                                             \
        AL(ptr, bytes);                                                              \
        if (hipMemsetAsync((ptr), 0, (bytes), s->stream) != hipSuccess) {            \
            bild_state_destroy(s);                                                   \
            return BILD_EHIP;                                                        \
        }                                                                            \
    } while (0)
        if (w == 0 && p->trunk_layers > 0) {
            // early-exit pair: the trunk's layers are the large model's first layers, one cache serves both
            // (filled in below, once the large model's buffers exist)
        } else {
            ALZ(M.kcache, L * (size_t)s->cap_len * I * esz);
            ALZ(M.vcache, L * (size_t)s->cap_len * I * esz);
            if (m->cfg.cross_attn) {
                ALZ(M.ck, L * (size_t)s->cap_src * I * esz);
                ALZ(M.cv, L * (size_t)s->cap_src * I * esz);
            }
        }
        // a decoder-only model prefills its whole prompt in one pass of many row blocks
        M.rows_cap = p->decoder_only ? std::max(kMaxRows, max_src) : kMaxRows;
        // the two residual-stream buffers in one block: a reader of partial results gets the other buffer as a 32-bit
        // offset from the one it reads (GemmArgs::x_out)
        AL(M.x, sizeof(float) * ((size_t)M.rows_cap + kMaxRows) * d);
        M.x2 = M.x + (size_t)M.rows_cap * d;
        AL(M.q, sizeof(float) * M.rows_cap * I);
        AL(M.a, sizeof(float) * M.rows_cap * I);
        AL(M.h, sizeof(float) * M.rows_cap * F);
        AL(M.px, sizeof(float) * kPartSlices * kMaxRows * d);
        if (d <= 1024) ALZ(M.pxh, sizeof(float) * kMaxHeadParts * kMaxRows * d);  // slots of heads a model does not have stay zero
        if (m->cfg.pos == BILD_POS_SINUSOIDAL) {
            AL(M.pe, sizeof(float) * (size_t)s->cap_len * d);
            if (launch_pe_table(M.pe, s->cap_len, (int)d, s->stream) != hipSuccess) {
                bild_state_destroy(s);
                return BILD_EHIP;
            }
        }
        if (m->cfg.dtype == BILD_DT_BF16) {
            AL(M.xb, sizeof(uint16_t) * 2 * kMaxRows * d);
            AL(M.ab, sizeof(uint16_t) * 2 * kMaxRows * I);
            AL(M.hb, sizeof(uint16_t) * 2 * kMaxRows * F);
            AL(M.ssq, sizeof(float) * (kMaxSsqParts + 8) * kMaxRows);
        }
        M.nparts_cap = (m->head.tn + 0) / 1 + 1;  // at most one partial per feature tile
        AL(M.part, sizeof(StatPart) * (size_t)M.nparts_cap * kMaxRows);
        AL(M.zt, sizeof(float) * kMaxRows);
        M.max_splits = std::max(8, std::min(64, (std::max(max_len, max_src) + 511) / 512));
        AL(M.att_o, sizeof(float) * (size_t)M.max_splits * kMaxRows * I);
        AL(M.att_ml, sizeof(float) * (size_t)M.max_splits * kMaxRows * m->cfg.n_heads * 2);
        if (m->cfg.n_enc_layers > 0) {
            AL(M.enc_x, sizeof(float) * (size_t)max_src * d);
            AL(M.enc_q, sizeof(float) * (size_t)max_src * I);
            AL(M.enc_a, sizeof(float) * (size_t)max_src * I);
            AL(M.enc_h, sizeof(float) * (size_t)max_src * F);
            ALZ(M.enc_k, (size_t)s->cap_src * I * esz);
            ALZ(M.enc_v, (size_t)s->cap_src * I * esz);
        }
    }
    if (p->trunk_layers > 0) {
        s->ms[0].kcache = s->ms[1].kcache;
        s->ms[0].vcache = s->ms[1].vcache;
        s->ms[0].ck = s->ms[1].ck;
        s->ms[0].cv = s->ms[1].cv;
        AL(s->trunk_x, sizeof(float) * (size_t)s->cap_len * p->m[1]->cfg.d_model);
    }
#undef ALZ
#undef AL
    if (hipMemsetAsync(s->ctl, 0, sizeof(Ctl), s->stream) != hipSuccess ||
        hipStreamSynchronize(s->stream) != hipSuccess) {
        bild_state_destroy(s);
        return BILD_EHIP;
    }
    *out = s;
    return BILD_OK;
}

namespace {

int push_ctl(bild_state* s) {
    Ctl* h = s->hctl;
    std::memset(h, 0, sizeof(Ctl));
    h->y_len = s->y_len;
    h->draft_start = s->draft_start;
    h->len[0] = s->len[0];
    h->len[1] = s->len[1];
    h->n_src = s->n_src;
    h->n_max = s->n_max;
    h->alpha_fb = s->alpha_fb;
    h->alpha_rb = s->alpha_rb;
    h->seq = s->seq_issued;
    HIPC(hipMemcpyAsync(s->ctl, h, sizeof(Ctl), hipMemcpyHostToDevice, s->stream));
    HIPC(hipStreamSynchronize(s->stream));
    return BILD_OK;
}

// Thresholds live in the device control block so that captured passes need no new arguments.
int set_alpha(bild_state* s, float fb, float rb) {
    // compare bit patterns so that +-inf and every other value round-trip exactly
    if (std::memcmp(&fb, &s->alpha_fb, 4) == 0 && std::memcmp(&rb, &s->alpha_rb, 4) == 0) return BILD_OK;
    HIPC(hipStreamSynchronize(s->stream));  // the staging buffer may still be in use by an earlier copy
    s->halpha[0] = fb;
    s->halpha[1] = rb;
    HIPC(hipMemcpyAsync(&s->ctl->alpha_fb, s->halpha, 8, hipMemcpyHostToDevice, s->stream));
    s->alpha_fb = fb;
    s->alpha_rb = rb;
    return BILD_OK;
}

// Waits for the last pass; its policy kernel has mirrored the control block into pinned host memory.  The mirror's pass
// counter is polled first (the kernel writes it last, behind a system-wide fence): that sees the result a few
// microseconds before the stream's completion reaches the host.  If the count does not arrive in time (a failed
// launch) the stream is waited for as usual and the two counts are brought together again.
int pull_ctl(bild_state* s) {
    bool seen = false;
    {
        const int* seq = &s->hctl->seq;
        const auto t0 = std::chrono::steady_clock::now();
        for (unsigned spins = 1;; ++spins) {
            // acquire: the other words of the mirror are read after the count that was written behind them
            if (__atomic_load_n(seq, __ATOMIC_ACQUIRE) == s->seq_issued) {
                seen = true;
                break;
            }
            if ((spins & 1023) == 0 && std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(500)) break;
        }
    }
    if (!seen) {
        HIPC(hipStreamSynchronize(s->stream));
        s->seq_issued = __atomic_load_n(&s->hctl->seq, __ATOMIC_ACQUIRE);
    }
    s->y_len = s->hctl->y_len;
    s->draft_start = s->hctl->draft_start;
    s->len[0] = s->hctl->len[0];
    s->len[1] = s->hctl->len[1];
    return BILD_OK;
}

}  // namespace

namespace bild {
// Key splits of one attention launch and whether the consumer projection merges them (`defer`).
// A workgroup's time grows with the K/V bytes it streams (about 2 us for 32 KiB, 3 us for 128 KiB, then in
// proportion).  Partials merged by the consumer cost no kernel: it works out the normalised weights once per
// (row, head) and then reads `splits` float4 per piece.  Measured on 512 keys of 64 dims, 24 layers: four
// splits of 32 KiB against none: 1055 / 1127 us per single-row pass, 1319 / 1351 us at 8 rows, 1585 / 1649 us at
// 16 rows, so the route is taken up to 16 rows (bounds: 8 splits, rows * heads <= 256, rows * heads * splits <= 1024
// - what the consumer's threads and its weight table in LDS hold).  The merge kernel costs about 5 us and therefore only pays when it
// brings a workgroup from above 160 KiB down to 128 KiB.
int pick_splits_raw(int d_head, int esz, int max_splits, int nkeys, int heads, int T, bool* defer) {
    const size_t per_head = (size_t)nkeys * d_head * 2 * esz;
    const size_t want = (size_t)(T <= 16 ? 32 : 128) << 10;
    auto fits = [&](int sp) { return sp <= max_splits && heads * sp <= 512; };
    int d_sp = 1;  // deferred route: as many splits as it allows, up to the wanted size
    // the consumer keeps one (row, head) pair per thread (at least 256 threads) and a table of splits x pairs
    // weights in the 4 KiB its smallest reduction area has
    const bool mergeable = T <= 16 && heads * T <= 256;
    while (per_head / d_sp > want && d_sp * 2 <= 8 && mergeable && heads * T * d_sp * 2 <= 1024 && fits(d_sp * 2)) d_sp *= 2;
    *defer = d_sp > 1;
    if (per_head / d_sp <= ((size_t)160 << 10)) return d_sp;
    int sp = d_sp;
    while (per_head / sp > ((size_t)128 << 10) && fits(sp * 2)) sp *= 2;
    if (sp > d_sp) *defer = false;
    return sp;
}

}  // namespace bild

namespace {

int pick_splits(const ModelState& M, int nkeys, int heads, int T, bool* defer) {
    return pick_splits_raw(M.m->cfg.d_head, M.m->esz(), M.max_splits, nkeys, heads, T, defer);
}

}  // namespace

namespace bild {

int pick_attn_waves(int dtype, int d_head, int T, int nkeys, int splits) {
    // one 32-key block per wave where possible, bounded by the LDS the merge needs
    const int blocks = ((nkeys + 31) / 32 + splits - 1) / splits;
    int nw = 1;
    while (nw < 8 && nw < blocks) nw *= 2;
    // at least four waves all the same: staging q is one piece per thread only from 256 threads on, and with fewer the
    // pieces are fetched one trip to memory after the other (measured: 1730 -> 1757 tokens/s on T5 shapes, whose caches
    // start short; eight waves cost more in the merge than they save)
    if (nw < 4) nw = 4;
    while (nw > 1 && attn_lds_bytes(dtype, d_head, T, nw) > 96 * 1024) nw /= 2;
    return nw;
}

}  // namespace bild

namespace {

GemmArgs gemm_base(const bild_model* m, const TMat& W, const float* x, int ldx, int T, const float* gain) {
    GemmArgs g;
    std::memset(&g, 0, sizeof(g));
    g.W = W;
    g.x = x;
    g.ldx = ldx;
    g.T = T;
    g.gain = gain;
    g.eps = m->cfg.norm_eps;
    g.d_head = m->cfg.d_head;
    g.i_dim = m->inner();
    g.rope_base = m->cfg.rope_base;
    g.act = m->cfg.act;
    g.vocab = m->cfg.vocab;
    return g;
}

int launch_gemm_profiled(bild_state* s, const bild_model* m, const GemmArgs& g) {
    s->gemm_count += 1;
    s->stage_count += 1;
    s->gemm_bytes += (int64_t)g.W.n * g.W.k * m->esz();
    if (!s->prof_on) {
        HIPC(launch_gemm(g, m->cfg.dtype, s->stream));
        return BILD_OK;
    }
    if (s->prof_used >= s->prof_cap) {
        s->prof_dropped++;
        HIPC(launch_gemm(g, m->cfg.dtype, s->stream));
        return BILD_OK;
    }
    const int i = s->prof_used++;
    HIPC(hipEventRecord(s->prof_ev[2 * i], s->stream));
    HIPC(launch_gemm(g, m->cfg.dtype, s->stream));
    HIPC(hipEventRecord(s->prof_ev[2 * i + 1], s->stream));
    bild_state::ProfRec r;
    r.model = (m == s->pair->m[1]) ? 1 : 0;
    r.cls = g.epi == EPI_LMHEAD ? 1 : 0;
    r.bytes = (int64_t)g.W.n * g.W.k * m->esz();
    s->prof_rec.push_back(r);
    return BILD_OK;
}

int run_gemm(bild_state* s, const bild_model* m, GemmArgs& g) {
    gemm_pick_shape(g, m->cfg.dtype);
    return launch_gemm_profiled(s, m, g);
}

int emit_gemm(bild_state* s, const bild_model* m, GemmArgs& g) {
    gemm_pick_shape(g, m->cfg.dtype);
    return launch_gemm_profiled(s, m, g);
}

// `deferred` receives the number of key splits whose partials the following output projection must merge
// (1: the attention output is complete).
int emit_attention(bild_state* s, const ModelState& M, AttnArgs& a, int nkeys, int* deferred) {
    const int dt = M.m->cfg.dtype;
    *deferred = 1;
    bool defer = false;
    a.splits = a.T > kMaxRows ? 1 : pick_splits(M, nkeys, a.heads, a.T, &defer);  // row blocks and key splits do not combine
    a.nw = pick_attn_waves(dt, a.d_head, std::min(a.T, kMaxRows), nkeys, a.splits);
    a.defer_merge = a.splits > 1 && defer;
    if (a.defer_merge) *deferred = a.splits;
    s->stage_count += (a.splits > 1 && !a.defer_merge) ? 2 : 1;  // (the merge kernel is a stage of its own)
    if (!s->gemm_only) HIPC(launch_attention(a, dt, s->stream));
    return BILD_OK;
}

// Embedding and all decoder layers of model w over rows y[len .. len+T).
int emit_layers(bild_state* s, int w, int T, int key_hint, bool head_reads_parts, int* xb_parts_out, float** x_out, bool* parts_pending) {
    ModelState& M = s->ms[w];
    const bild_model* m = M.m;
    const bild_model_config& c = m->cfg;
    const int d = c.d_model, I = m->inner(), F = c.d_ff, dt = c.dtype;
    const size_t esz = m->esz();
    const int* len_ptr = &s->ctl->len[w];
    EmbedArgs e;
    std::memset((void*)&e, 0, sizeof(e));
    e.E = m->emb;
    e.tokens = s->y;
    e.base_ptr = len_ptr;
    e.T = T;
    e.d = d;
    e.vocab = c.vocab;
    e.tie_shift = c.tie_shift;
    e.sinusoidal = c.pos == BILD_POS_SINUSOIDAL;
    e.embed_scale = c.embed_scale;
    e.x = M.x;
    e.pe = M.pe;
    // Early-exit pair: the large model's pass starts from the hidden state the trunk (model 0) left for these
    // rows and runs the layers above the trunk only.
    const int trunk = s->pair->trunk_layers;
    const bool above_trunk = trunk > 0 && w == 1;
    const int layer0 = above_trunk ? trunk : 0;
    // Passes of a few rows of a bf16 model: every producer leaves its output as high / low bf16 planes for the
    // projection that follows (x times that projection's norm gain, the attention output, the FFN hidden state).
    // Measured (us per large-model pass, planes / fp32 hand-over): 1024-wide model 2 rows 1002 / 947, 5 rows 1121 / 1148,
    // 16 rows 1332 / 1429, 32 rows 1831 / 2018; 4096-wide model 2 rows 3398 / 3487, 11 rows 3904 / 4326, 32 rows 5321 / 6384.
    // Below five rows the narrow models keep the kernels specialised for one and for two to four rows.
    const int planes_from = s->pre_min_rows > 0 ? s->pre_min_rows : (d >= 2048 ? 2 : 5);
    const bool planes = dt == BILD_DT_BF16 && T >= planes_from && T <= kMaxRows && M.xb != nullptr;
    uint16_t *xb_hi = M.xb, *xb_lo = M.xb ? M.xb + (size_t)kMaxRows * d : nullptr;
    uint16_t *ab_hi = M.ab, *ab_lo = M.ab ? M.ab + (size_t)kMaxRows * I : nullptr;
    uint16_t *hb_hi = M.hb, *hb_lo = M.hb ? M.hb + (size_t)kMaxRows * F : nullptr;
    int xb_parts = 0;  // > 0: xb holds the current residual stream, with this many partial sums of squares in M.ssq
    // the norm gain in front of the projection that reads the residual stream next
    auto set_in = [&](GemmArgs& g) {  // input from the residual-stream planes, if they are current
        if (xb_parts > 0) { g.xb_hi = xb_hi; g.xb_lo = xb_lo; g.ssq_part = M.ssq; g.ssq_parts = xb_parts; }
    };
    auto set_out = [&](GemmArgs& g, const float* next_gain) {  // residual epilogue: also planes for the next projection
        if (!planes) return;
        g.nx_hi = xb_hi; g.nx_lo = xb_lo; g.nx_gain = next_gain; g.nx_ssq = M.ssq; g.nx_ld = d;
    };
    auto after_out = [&](const GemmArgs& g) {  // (after gemm_pick_shape) one partial per wave that owns output tiles
        xb_parts = planes ? (int)gemm_num_blocks(g) * (g.nwv / g.wk) : 0;
        if (xb_parts > kMaxSsqParts) xb_parts = 0;  // more than a consumer adds up: the next projection converts x itself
    };
    // The FFN output projection of a narrow model at one to four rows (64 feature tiles x thousands of inputs: too few
    // workgroups with too long a stream each) is cut into kPartSlices slices of its inputs; the next layer's first
    // projection (or the LM head of a single-row pass) adds the slices to the residual stream while staging and leaves the
    // sum in the other of two residual buffers.  Measured on the T5-large shape: see the design notes.
    const int kt = dt == BILD_DT_BF16 ? 32 : 16;
    const bool split_ffn = !planes && T <= 4 && d <= s->ksplit_max_d && s->ksplit_min_f > 0 && F >= s->ksplit_min_f &&
                           (F / kt) % kPartSlices == 0 && (T == 1 || ((d / 4) % 64 == 0 && (F / kPartSlices / 4) % 64 == 0)) && M.px != nullptr;
    float *xcur = M.x, *xoth = M.x2;
    // > 0: the residual stream is xcur + that many partial results in pend_buf (slices of a split FFN output projection,
    // or one per head of an attention fused with its output projection), to be added by the next reader
    int pending = 0;
    const float* pend_buf = nullptr;
    auto set_parts_in = [&](GemmArgs& g) {
        if (!pending) return;
        g.px = pend_buf; g.px_stride = (int64_t)kMaxRows * d; g.pn = pending; g.x_out = xoth;
    };
    auto after_parts_in = [&]() {
        if (!pending) return;
        std::swap(xcur, xoth);
        pending = 0;
    };
    // Single-row passes of the narrow models: attention and its output projection as one kernel per (head, column
    // group); the next projection adds one partial result per head.  A head's cache must be small enough for one
    // workgroup (every column group repeats the head's attention).
    const bool fuse_shape = s->fuse_attn && T == 1 && !planes && d <= 1024 && c.n_heads <= kMaxHeadParts && c.d_head <= 64 &&
                            c.d_head % kt == 0 && M.pxh != nullptr;
    auto fuse_attention = [&](AttnArgs& a, const TMat& wo, int nkeys) -> int {  // 1: launched fused, 0: not applicable, < 0: error
        // (measured on the T5-large shape: 64 keys 6.1 us against 4.7 + 3.5 for attention and projection apart; 512 keys,
        // 128 KiB per head, 11.3 us against 5.1 + 4.5)
        if (!fuse_shape || (size_t)nkeys * c.d_head * 2 * esz > (size_t)s->fuse_max_kv) return 0;
        a.splits = 1;
        a.defer_merge = 0;
        a.nw = pick_attn_waves(dt, a.d_head, T, nkeys, 1);
        const int maxn = dt == BILD_DT_BF16 ? 4 : 2;
        int cg = std::max(1, std::min(wo.tn, 64 / c.n_heads));
        while (cg < wo.tn && ((wo.tn + cg - 1) / cg + a.nw - 1) / a.nw > maxn) cg *= 2;
        if (((wo.tn + cg - 1) / cg + a.nw - 1) / a.nw > maxn) return 0;
        a.wo = wo;
        a.proj_out = M.pxh;
        a.proj_stride = (int64_t)kMaxRows * d;
        a.cgroups = cg;
        a.d_model = d;
        s->stage_count += 1;
        if (!s->gemm_only && launch_attention_proj(a, dt, s->stream) != hipSuccess) return BILD_EHIP;
        pending = kMaxHeadParts;
        pend_buf = M.pxh;
        return 1;
    };
    if (planes && !above_trunk) {
        e.nx_hi = xb_hi; e.nx_lo = xb_lo; e.nx_gain = m->dec[layer0].ln1; e.nx_ssq = M.ssq;
        xb_parts = kEmbedSsqParts;
    }
    // Single-row passes: the first projection gathers the row from the embedding matrix itself (no embedding kernel).
    // The table of positions must exist where positions are added (the kernel does not evaluate sines).
    // Every workgroup of that projection repeats the gather, so it is taken only where one round of two pieces per
    // thread covers the row (a 4096-wide row in workgroups of two waves would be four dependent rounds: measured slower).
    bool embed_in_proj = s->fuse_embed && T == 1 && !planes && !above_trunk && (!e.sinusoidal || e.pe != nullptr) &&
                         c.tie_shift >= 0 && c.tie_shift < c.vocab && layer0 < c.n_dec_layers;
    if (embed_in_proj) {
        GemmArgs probe = gemm_base(m, m->dec[layer0].wqkv, M.x, d, T, m->dec[layer0].ln1);
        probe.epi = EPI_QKV;
        gemm_pick_shape(probe, dt);
        embed_in_proj = d / 4 <= 2 * 64 * probe.nwv && probe.W.k <= probe.kc;
    }
    if (!embed_in_proj) s->stage_count += 1;  // embedding or the trunk's rows
    if (!s->gemm_only && !embed_in_proj) {
        if (above_trunk) {
            RowCopyArgs rc;
            std::memset((void*)&rc, 0, sizeof(rc));
            rc.src = s->trunk_x;
            rc.src_row_ptr = len_ptr;
            rc.dst = M.x;
            rc.d = d;
            rc.T = T;
            HIPC(launch_row_copy(rc, s->stream));
        } else {
            HIPC(launch_embed(e, dt, s->stream));
        }
    }
    const float att_scale = 1.f / std::sqrt((float)c.d_head);
    int merge_splits = 1;
    for (int l = layer0; l < c.n_dec_layers; ++l) {
        const LayerW& L = m->dec[l];
        char* kc = M.kcache + (size_t)l * s->cap_len * I * esz;
        char* vc = M.vcache + (size_t)l * s->cap_len * I * esz;
        int fused = 0;  // this attention ran together with its output projection
        {
            GemmArgs g = gemm_base(m, L.wqkv, xcur, d, T, L.ln1);
            set_parts_in(g);
            g.epi = EPI_QKV;
            g.q_dim = I;
            g.q_out = M.q;
            g.k_cache = kc;
            g.v_cache = vc;
            g.vcap = s->cap_len;
            g.pos_ptr = len_ptr;
            g.rope = c.pos == BILD_POS_ROPE;
            set_in(g);
            if (embed_in_proj && l == layer0) {
                g.e_w = e.E.w; g.e_tk = e.E.tk; g.e_tokens = e.tokens; g.e_base_ptr = e.base_ptr; g.e_base_add = e.base_add;
                g.e_vocab = e.vocab; g.e_shift = e.tie_shift; g.e_scale = e.embed_scale; g.e_pe = e.sinusoidal ? e.pe : nullptr;
                g.x_out = xcur;  // (= g.x: the row is written where the embedding kernel would have left it)
            }
            int rc = emit_gemm(s, m, g);
            if (rc) return rc;
            after_parts_in();
        }
        {
            AttnArgs a;
            std::memset((void*)&a, 0, sizeof(a));
            a.q = M.q; a.k = kc; a.v = vc; a.out = M.a;
            a.T = T; a.heads = c.n_heads; a.d_head = c.d_head; a.i_dim = I;
            a.causal = 1;
            a.len_ptr = len_ptr;
            a.rel_bias = m->dec_rel;
            a.rel_d = c.rel_max_dist;
            a.vcap = s->cap_len;
            a.part_o = M.att_o; a.part_ml = M.att_ml;
            a.scale = att_scale;
            if (planes) { a.ob_hi = ab_hi; a.ob_lo = ab_lo; }
            fused = fuse_attention(a, L.wo, key_hint);
            if (fused < 0) return fused;
            if (!fused) {
                int rc = emit_attention(s, M, a, key_hint, &merge_splits);
                if (rc) return rc;
            }
        }
        if (!fused) {
            GemmArgs g = gemm_base(m, L.wo, M.a, I, T, nullptr);
            g.epi = EPI_RESID;
            g.out = xcur;
            g.ldo = d;
            if (merge_splits > 1) { g.mg_splits = merge_splits; g.mg_o = M.att_o; g.mg_ml = M.att_ml; g.mg_heads = c.n_heads; }
            else if (planes) { g.xb_hi = ab_hi; g.xb_lo = ab_lo; }
            set_out(g, c.cross_attn ? L.lnc : L.ln2);
            int rc = emit_gemm(s, m, g);
            if (rc) return rc;
            after_out(g);
        }
        if (c.cross_attn) {
            {
                GemmArgs g = gemm_base(m, L.cwq, xcur, d, T, L.lnc);
                g.epi = EPI_STORE;
                g.out = M.q;
                g.ldo = I;
                set_in(g);
                set_parts_in(g);
                int rc = emit_gemm(s, m, g);
                if (rc) return rc;
                after_parts_in();
            }
            {
                AttnArgs a;
                std::memset((void*)&a, 0, sizeof(a));
                a.q = M.q;
                a.k = M.ck + (size_t)l * s->cap_src * I * esz;
                a.v = M.cv + (size_t)l * s->cap_src * I * esz;
                a.vcap = s->cap_src;
                a.out = M.a;
                a.T = T; a.heads = c.n_heads; a.d_head = c.d_head; a.i_dim = I;
                a.causal = 0;
                a.len_ptr = &s->ctl->n_src;
                a.part_o = M.att_o; a.part_ml = M.att_ml;
                a.scale = att_scale;
                if (planes) { a.ob_hi = ab_hi; a.ob_lo = ab_lo; }
                fused = fuse_attention(a, L.cwo, s->n_src);
                if (fused < 0) return fused;
                if (!fused) {
                    int rc = emit_attention(s, M, a, s->n_src, &merge_splits);
                    if (rc) return rc;
                }
            }
            if (!fused) {
                GemmArgs g = gemm_base(m, L.cwo, M.a, I, T, nullptr);
                g.epi = EPI_RESID;
                g.out = xcur;
                g.ldo = d;
                if (merge_splits > 1) { g.mg_splits = merge_splits; g.mg_o = M.att_o; g.mg_ml = M.att_ml; g.mg_heads = c.n_heads; }
                else if (planes) { g.xb_hi = ab_hi; g.xb_lo = ab_lo; }
                set_out(g, L.ln2);
                int rc = emit_gemm(s, m, g);
                if (rc) return rc;
                after_out(g);
            }
        }
        {
            GemmArgs g = gemm_base(m, L.win, xcur, d, T, L.ln2);
            g.epi = EPI_ACT;
            g.out = M.h;
            g.ldo = F;
            set_in(g);
            set_parts_in(g);
            // the hidden state goes on as planes only if this projection itself reads planes (one kernel family per pass)
            const bool h_planes = planes && g.xb_hi != nullptr;
            if (h_planes) { g.nx_hi = hb_hi; g.nx_lo = hb_lo; g.nx_ld = F; }
            int rc = emit_gemm(s, m, g);
            if (rc) return rc;
            after_parts_in();
            GemmArgs g2 = gemm_base(m, L.wout, M.h, F, T, nullptr);
            g2.epi = EPI_RESID;
            g2.out = xcur;
            g2.ldo = d;
            if (split_ffn && (l + 1 < c.n_dec_layers || head_reads_parts)) {
                g2.epi = EPI_PART;
                g2.out = M.px;
                g2.ksplit = kPartSlices;
                g2.part_stride = (int64_t)kMaxRows * d;
                pending = kPartSlices;
                pend_buf = M.px;
            }
            if (h_planes) { g2.xb_hi = hb_hi; g2.xb_lo = hb_lo; }
            // the next reader of the residual stream: the following layer's first norm, or the final norm (LM head)
            if (h_planes) set_out(g2, l + 1 < c.n_dec_layers ? m->dec[l + 1].ln1 : m->dec_final);
            rc = emit_gemm(s, m, g2);
            if (rc) return rc;
            if (h_planes) after_out(g2); else xb_parts = 0;
        }
    }
    if (trunk > 0 && w == 0) s->stage_count += 1;
    if (trunk > 0 && w == 0 && !s->gemm_only) {  // remember what the trunk produced for these positions
        RowCopyArgs rc;
        std::memset((void*)&rc, 0, sizeof(rc));
        rc.src = xcur;
        rc.dst = s->trunk_x;
        rc.dst_row_ptr = len_ptr;
        rc.d = d;
        rc.T = T;
        HIPC(launch_row_copy(rc, s->stream));
    }
    *xb_parts_out = xb_parts;
    *x_out = xcur;
    *parts_pending = pending > 0;
    return BILD_OK;
}

}  // namespace

namespace bild {

// One decoder pass of model w over rows y[len .. len+T): embed, layers, and (lm_rows > 0)
// the LM head over the last lm_rows rows followed by the policy `mode`; lm_rows == 0
// only advances the cache (catch-up / prefill).
int decoder_pass(bild_state* s, int w, int T, int lm_rows, int mode, int key_hint) {
    ModelState& M = s->ms[w];
    const bild_model* m = M.m;
    const bild_model_config& c = m->cfg;
    const int d = c.d_model, dt = c.dtype;
    const int* len_ptr = &s->ctl->len[w];
    s->stage_count = 0;
    int xb_parts = 0;  // > 0: the final hidden state also sits in M.xb as bf16 planes (times the final norm's gain)
    float* xfin = M.x;  // the residual stream after the last layer ...
    bool parts = false; // ... to which the partial results in M.px are still to be added (split FFN output projection)
    {
        // a single-row pass whose LM head is the one-row kernel with one feature tile per wave can add them itself
        const bool head_reads_parts = T == 1 && lm_rows == 1 && s->pair->trunk_layers == 0 && m->head.tn < 8192;
        int rc = emit_layers(s, w, T, key_hint, head_reads_parts, &xb_parts, &xfin, &parts);
        if (rc) return rc;
    }
    FinishArgs f;
    std::memset((void*)&f, 0, sizeof(f));
    f.ctl = s->ctl;
    f.y = s->y;
    f.which = w;
    f.rows_consumed = T;
    f.y_cap = s->max_len;
    f.host_mirror = s->hctl_dev;
    if (lm_rows > 0) {
        GemmArgs g = gemm_base(m, m->head, xfin + (size_t)(T - lm_rows) * d, d, lm_rows, m->dec_final);
        if (parts) { g.px = M.px; g.px_stride = (int64_t)kMaxRows * d; g.pn = kPartSlices; g.x_out = xfin == M.x ? M.x2 : M.x; }
        g.epi = EPI_LMHEAD;
        g.scale = c.logit_scale;
        g.pos_ptr = len_ptr;
        g.pos_add = T - lm_rows;
        g.y = s->y;
        g.ylen_ptr = &s->ctl->y_len;
        g.part = M.part;
        g.zt = M.zt;
        g.dbg = (s->debug_logits || s->top_p > 0.f) ? M.dbg : nullptr;  // the draw of the sampling variant reads the logits
        g.row_off = 0;
        if (xb_parts > 0) {
            g.xb_hi = M.xb + (size_t)(T - lm_rows) * d;
            g.xb_lo = M.xb + (size_t)kMaxRows * d + (size_t)(T - lm_rows) * d;
            g.ssq_part = M.ssq + (T - lm_rows);
            g.ssq_parts = xb_parts;
        }
        gemm_pick_shape(g, dt);
        if ((int)gemm_num_blocks(g) > M.nparts_cap) return BILD_ECAP;
        {
            int rc = launch_gemm_profiled(s, m, g);
            if (rc) return rc;
        }
        f.part = M.part;
        f.nparts = (int)gemm_num_blocks(g);
        f.zt = M.zt;
        f.T = lm_rows;
        f.mode = mode;
        if (s->top_p > 0.f) {
            f.top_p = s->top_p;
            f.logits = M.dbg;
            f.vocab = c.vocab;
            f.u = s->u_dev[w];
            if (s->accept_mode == 1) {
                f.accept_mode = 1;
                f.u_acc = s->u_acc;
                f.s_ring = s->s_ring;
                f.s_draw = s->s_draw;
            }
        }
    } else {
        f.mode = 3;
    }
    // sampling variant under the threshold rule: the draw runs spread over the chip (seven launches instead of one)
    const bool spread = f.top_p > 0.f && f.mode <= 2 && f.accept_mode == 0 && s->draw_spread && s->draw_ws &&
                        c.vocab <= kDrawSliceIds * kDrawMaxSlices;
    s->stage_count += spread ? kFinishDrawStages : 1;
    if (spread) f.dws = s->draw_ws;
    if (!s->gemm_only) HIPC(spread ? launch_finish_draw(f, s->stream) : launch_finish(f, s->stream));
    return BILD_OK;
}

int key_bucket(int nkeys) {
    int b = 64;
    while (b < nkeys) b *= 2;
    return b;
}

// One pass, replayed from a captured graph when possible.  Launch parameters that depend on the cache
// length are chosen per power-of-two bucket of the key count, so a graph stays valid while the
// sequence grows inside its bucket; everything else the kernels need they read from the control block.
int run_pass(bild_state* s, int w, int T, int lm_rows, int mode) {
    if (s->pair->trunk_layers > 0 && w == 1 && s->len[0] < s->len[1] + T) {
        // early-exit pair: the upper layers continue from what the trunk left for these rows
        const int rc = catch_up(s, 0, s->len[1] + T);
        if (rc) return rc;
    }
    const int bucket = key_bucket(s->len[w] + T);
    if (lm_rows > 0) s->ms[w].last_rows = lm_rows;
    if (!s->use_graphs || s->prof_on || mode == 3) {
        const int rc = decoder_pass(s, w, T, lm_rows, mode, bucket);
        if (rc == BILD_OK && !s->gemm_only) s->seq_issued += 1;  // its policy kernel will count this pass
        return rc;
    }
    const std::array<int, 6> key = {w, T, lm_rows, mode, bucket, (s->debug_logits ? 1 : 0) | (s->gemm_only ? 2 : 0) | (s->top_p > 0.f ? 4 : 0) | (s->accept_mode ? 8 : 0)};
    auto it = s->graphs.find(key);
    if (it == s->graphs.end()) {
        hipGraph_t g = nullptr;
        HIPC(hipStreamBeginCapture(s->stream, hipStreamCaptureModeThreadLocal));
        const int rc = decoder_pass(s, w, T, lm_rows, mode, bucket);
        const hipError_t e = hipStreamEndCapture(s->stream, &g);
        if (rc != BILD_OK || e != hipSuccess) {
            if (g) (void)hipGraphDestroy(g);
            return rc != BILD_OK ? rc : BILD_EHIP;
        }
        hipGraphExec_t ge = nullptr;
        const hipError_t e2 = hipGraphInstantiate(&ge, g, nullptr, nullptr, 0);
        (void)hipGraphDestroy(g);
        if (e2 != hipSuccess) return BILD_EHIP;
        it = s->graphs.emplace(key, ge).first;
    }
    HIPC(hipGraphLaunch(it->second, s->stream));
    if (!s->gemm_only) s->seq_issued += 1;
    return BILD_OK;
}

// Brings model w's cache up to `target` consumed rows with LM-head-less passes.
int catch_up(bild_state* s, int w, int target) {
    while (s->len[w] < target) {
        const int T = std::min(s->ms[w].rows_cap, target - s->len[w]);
        int rc = run_pass(s, w, T, 0, 3);
        if (rc) return rc;
        s->len[w] += T;  // the device advances the same amount
    }
    return BILD_OK;
}

}  // namespace bild

namespace {

// Encoder of model w over the source in s->src, then the cross K/V of every decoder
// layer of each model that uses this encoder's output.
int run_encoder(bild_state* s, int w) {
    ModelState& M = s->ms[w];
    const bild_model* m = M.m;
    const bild_model_config& c = m->cfg;
    const int d = c.d_model, I = m->inner(), F = c.d_ff, dt = c.dtype, S = s->n_src;
    const float att_scale = 1.f / std::sqrt((float)c.d_head);
    // every launch covers all S source rows (row blocks of kMaxRows inside the kernels)
    {
        EmbedArgs e;
        std::memset((void*)&e, 0, sizeof(e));
        e.E = m->emb; e.tokens = s->src; e.T = S; e.d = d; e.vocab = c.vocab;
        e.tie_shift = c.tie_shift; e.sinusoidal = c.pos == BILD_POS_SINUSOIDAL; e.embed_scale = c.embed_scale;
        e.x = M.enc_x;
        HIPC(launch_embed(e, dt, s->stream));
    }
    for (int l = 0; l < c.n_enc_layers; ++l) {
        const LayerW& L = m->enc[l];
        {
            GemmArgs g = gemm_base(m, L.wqkv, M.enc_x, d, S, L.ln1);
            g.epi = EPI_QKV;
            g.q_dim = I;
            g.q_out = M.enc_q;
            g.k_cache = M.enc_k;
            g.v_cache = M.enc_v;
            g.vcap = s->cap_src;
            g.rope = c.pos == BILD_POS_ROPE;
            int rc = run_gemm(s, m, g);
            if (rc) return rc;
        }
        {
            AttnArgs a;
            std::memset((void*)&a, 0, sizeof(a));
            a.q = M.enc_q; a.k = M.enc_k; a.v = M.enc_v; a.out = M.enc_a;
            a.T = S; a.heads = c.n_heads; a.d_head = c.d_head; a.i_dim = I;
            a.causal = 0;
            a.nkeys_fixed = S;
            a.rel_bias = m->enc_rel;
            a.rel_d = c.rel_max_dist;
            a.len_ptr = &s->ctl->n_src;  // not used with a fixed count, but the kernel reads it
            a.vcap = s->cap_src;
            a.splits = 1;
            a.nw = pick_attn_waves(dt, c.d_head, std::min(S, kMaxRows), S, 1);
            a.scale = att_scale;
            HIPC(launch_attention(a, dt, s->stream));
        }
        {
            GemmArgs g = gemm_base(m, L.wo, M.enc_a, I, S, nullptr);
            g.epi = EPI_RESID;
            g.out = M.enc_x;
            g.ldo = d;
            int rc = run_gemm(s, m, g);
            if (rc) return rc;
        }
        {
            GemmArgs g = gemm_base(m, L.win, M.enc_x, d, S, L.ln2);
            g.epi = EPI_ACT;
            g.out = M.enc_h;
            g.ldo = F;
            int rc = run_gemm(s, m, g);
            if (rc) return rc;
        }
        {
            GemmArgs g = gemm_base(m, L.wout, M.enc_h, F, S, nullptr);
            g.epi = EPI_RESID;
            g.out = M.enc_x;
            g.ldo = d;
            int rc = run_gemm(s, m, g);
            if (rc) return rc;
        }
    }
    // cross K/V: K = norm_final(enc_x) Wk, V = ... for this model and, if it borrows, the small one
    for (int u = 0; u < 2; ++u) {
        const bool uses = (u == w) || (u == 0 && w == 1 && s->pair->small_borrows_encoder);
        if (!uses) continue;
        if (u == 0 && s->pair->trunk_layers > 0) continue;  // a view of the large model: the same cross K/V memory
        ModelState& U = s->ms[u];
        const bild_model* mu = U.m;
        const int Iu = mu->inner();
        const size_t esz = mu->esz();
        for (int l = 0; l < mu->cfg.n_dec_layers; ++l) {
            GemmArgs g = gemm_base(mu, mu->dec[l].cwkv, M.enc_x, d, S, m->enc_final);
            g.eps = m->cfg.norm_eps;
            g.epi = EPI_QKV;
            g.q_dim = 0;
            g.i_dim = Iu;
            g.k_cache = U.ck + (size_t)l * s->cap_src * Iu * esz;
            g.v_cache = U.cv + (size_t)l * s->cap_src * Iu * esz;
            g.vcap = s->cap_src;
            g.rope = 0;
            int rc = run_gemm(s, mu, g);
            if (rc) return rc;
        }
    }
    return BILD_OK;
}

}  // namespace

// ======================================================================= request API
extern "C" int bild_encode(bild_state* s, const int32_t* src, int n_src) {
    if (!s || !src) return BILD_EINVAL;
    if (n_src < 1) return BILD_EINVAL;
    if (n_src > s->max_src) return BILD_ECAP;
    const int V = s->pair->m[1]->cfg.vocab;
    for (int i = 0; i < n_src; ++i)
        if (src[i] < 0 || src[i] >= V) return BILD_EINVAL;
    const bool dec_only = s->pair->decoder_only;
    if (dec_only && n_src + 1 > s->max_len) return BILD_ECAP;
    s->encoded = false;
    s->n_src = n_src;
    s->len[0] = s->len[1] = 0;
    if (dec_only) {
        HIPC(hipMemcpyAsync(s->y, src, sizeof(int) * (size_t)n_src, hipMemcpyHostToDevice, s->stream));
        s->y_len = n_src;
    } else {
        const int32_t bos = s->pair->m[1]->cfg.bos;
        HIPC(hipMemcpyAsync(s->src, src, sizeof(int) * (size_t)n_src, hipMemcpyHostToDevice, s->stream));
        HIPC(hipMemcpyAsync(s->y, &bos, sizeof(int), hipMemcpyHostToDevice, s->stream));
        s->y_len = 1;
    }
    s->n0 = s->y_len;
    s->draft_start = s->y_len;
    int rc = push_ctl(s);
    if (rc) return rc;
    if (dec_only) {
        for (int w = 0; w < 2; ++w) {
            rc = catch_up(s, w, n_src - 1);
            if (rc) return rc;
        }
    } else {
        rc = run_encoder(s, 1);
        if (rc) return rc;
        if (!s->pair->small_borrows_encoder) {
            rc = run_encoder(s, 0);
            if (rc) return rc;
        }
    }
    HIPC(hipStreamSynchronize(s->stream));  // the encoder's kernels end with no policy kernel: wait for the stream itself
    rc = pull_ctl(s);
    if (rc) return rc;
    s->encoded = true;
    return BILD_OK;
}

extern "C" int bild_small_step(bild_state* s, float alpha_fb, int32_t* token, int32_t* fallback_flag,
                               float* max_prob) {
    if (!s || !token || !fallback_flag) return BILD_EINVAL;
    if (!s->encoded) return BILD_ESTATE;
    if (s->len[0] >= s->y_len) return BILD_ESTATE;  // nothing unconsumed
    if (s->y_len >= s->max_len) return BILD_ECAP;
    int rc = set_alpha(s, alpha_fb, s->alpha_rb);
    if (rc) return rc;
    rc = catch_up(s, 0, s->y_len - 1);
    if (rc) return rc;
    rc = run_pass(s, 0, 1, 1, 0);
    if (rc) return rc;
    rc = pull_ctl(s);
    if (rc) return rc;
    *token = s->hctl->res_tok;
    *fallback_flag = s->hctl->res_flag & 1;
    if (max_prob) *max_prob = s->hctl->res_pmax;
    return BILD_OK;
}

extern "C" int bild_large_verify(bild_state* s, const int32_t* draft, int n, float alpha_rb, int32_t* out_tokens,
                                 int32_t* n_out, int32_t* rollback_pos, float* nll) {
    if (!s || !out_tokens || !n_out || !rollback_pos) return BILD_EINVAL;
    if (!s->encoded) return BILD_ESTATE;
    if (draft) {
        if (n < 0) return BILD_EINVAL;
        if (n + 1 > kMaxRows) return BILD_ECAP;
        if (s->draft_start + n + 1 > s->max_len) return BILD_ECAP;
        const int V = s->pair->m[1]->cfg.vocab;
        for (int i = 0; i < n; ++i)
            if (draft[i] < 0 || draft[i] >= V) return BILD_EINVAL;
        if (n > 0)
            HIPC(hipMemcpyAsync(s->y + s->draft_start, draft, sizeof(int) * (size_t)n, hipMemcpyHostToDevice,
                                s->stream));
        s->y_len = s->draft_start + n;
        s->len[0] = std::min(s->len[0], s->draft_start);
        s->len[1] = std::min(s->len[1], s->draft_start - 1);
        int rc = push_ctl(s);
        if (rc) return rc;
    } else {
        n = s->y_len - s->draft_start;
        if (n + 1 > kMaxRows) return BILD_ECAP;
        if (s->y_len + 1 > s->max_len) return BILD_ECAP;
    }
    if (s->len[1] > s->draft_start - 1) return BILD_ESTATE;
    int rc = set_alpha(s, s->alpha_fb, alpha_rb);
    if (rc) return rc;
    rc = catch_up(s, 1, s->draft_start - 1);
    if (rc) return rc;
    const int ds = s->draft_start;
    rc = run_pass(s, 1, n + 1, n + 1, 1);
    if (rc) return rc;
    rc = pull_ctl(s);
    if (rc) return rc;
    const int r = s->hctl->res_r;
    *rollback_pos = r;
    *n_out = r + 1;
    HIPC(hipMemcpyAsync(out_tokens, s->y + ds, sizeof(int) * (size_t)(r + 1), hipMemcpyDeviceToHost, s->stream));
    HIPC(hipStreamSynchronize(s->stream));
    if (nll)
        for (int i = 0; i < n; ++i) nll[i] = (i <= r) ? s->hctl->res_nll[i] : NAN;
    return BILD_OK;
}

extern "C" int bild_kv_truncate(bild_state* s, int which, int pos) {
    if (!s || which < 1 || which > 3 || pos < 0) return BILD_EINVAL;
    if (!s->encoded) return BILD_ESTATE;
    if ((which & 1) && pos > s->len[0]) return BILD_EINVAL;
    if ((which & 2) && pos > s->len[1]) return BILD_EINVAL;
    // the large model must never be ahead of draft_start - 1; cutting only lowers lengths
    if (which & 1) s->len[0] = pos;
    if (which & 2) s->len[1] = pos;
    return push_ctl(s);
}

extern "C" int bild_seq_truncate(bild_state* s, int n_keep) {
    if (!s) return BILD_EINVAL;
    if (!s->encoded) return BILD_ESTATE;
    if (n_keep < s->n0 || n_keep > s->y_len) return BILD_EINVAL;
    s->y_len = n_keep;
    s->draft_start = std::min(s->draft_start, n_keep);
    s->len[0] = std::min(s->len[0], n_keep - 1);
    s->len[1] = std::min(s->len[1], s->draft_start - 1);
    return push_ctl(s);
}

extern "C" int bild_force_tokens(bild_state* s, int first, const int32_t* tokens, int n, int draft_start) {
    if (!s || n < 0 || (n > 0 && !tokens)) return BILD_EINVAL;
    if (!s->encoded) return BILD_ESTATE;
    if (first < s->n0 || first > s->y_len) return BILD_EINVAL;
    if (first + n >= s->max_len) return BILD_ECAP;
    if (draft_start < s->n0 || draft_start > first + n) return BILD_EINVAL;
    const int V = s->pair->m[1]->cfg.vocab;
    for (int i = 0; i < n; ++i)
        if (tokens[i] < 0 || tokens[i] >= V) return BILD_EINVAL;
    if (n > 0)
        HIPC(hipMemcpyAsync(s->y + first, tokens, sizeof(int) * (size_t)n, hipMemcpyHostToDevice, s->stream));
    s->y_len = first + n;
    s->draft_start = draft_start;
    s->len[0] = std::min(s->len[0], first);
    s->len[1] = std::min(s->len[1], std::min(first, draft_start - 1));
    return push_ctl(s);
}

extern "C" int bild_get_lengths(bild_state* s, int32_t* y_len, int32_t* draft_start, int32_t* len_small,
                                int32_t* len_large) {
    if (!s) return BILD_EINVAL;
    if (y_len) *y_len = s->y_len;
    if (draft_start) *draft_start = s->draft_start;
    if (len_small) *len_small = s->len[0];
    if (len_large) *len_large = s->len[1];
    return BILD_OK;
}

extern "C" int bild_get_sequence(bild_state* s, int32_t* out, int cap, int32_t* n) {
    if (!s || !out || !n) return BILD_EINVAL;
    if (cap < s->y_len) return BILD_ECAP;
    if (s->y_len > 0) {
        HIPC(hipMemcpyAsync(out, s->y, sizeof(int) * (size_t)s->y_len, hipMemcpyDeviceToHost, s->stream));
        HIPC(hipStreamSynchronize(s->stream));
    }
    *n = s->y_len;
    return BILD_OK;
}

extern "C" int bild_generate(bild_state* s, const int32_t* src, int n_src, float alpha_fb, float alpha_rb,
                             int max_new, int32_t eos, int32_t* out, int32_t* n_out, bild_stats* stats) {
    if (!s || !out || !n_out || max_new < 0) return BILD_EINVAL;
    int rc = BILD_OK;
    if (src) {
        rc = bild_encode(s, src, n_src);
        if (rc) return rc;
    } else if (!s->encoded) {
        return BILD_ESTATE;
    }
    if (s->n0 + max_new > s->max_len) return BILD_ECAP;
    bild_stats st;
    std::memset(&st, 0, sizeof(st));
    int last = -1;
    while (s->y_len - s->n0 < max_new && !(s->y_len > s->n0 && last == eos && eos >= 0)) {
        int32_t tok, flag;
        rc = bild_small_step(s, alpha_fb, &tok, &flag, nullptr);
        if (rc) return rc;
        st.small_steps++;
        if (!flag) {
            last = tok;
            continue;
        }
        if (s->hctl->res_flag & 2)
            st.fallbacks_forced++;
        else
            st.fallbacks_conf++;
        int32_t toks[kMaxRows], cnt, r;
        const int n = s->y_len - s->draft_start;
        rc = bild_large_verify(s, nullptr, 0, alpha_rb, toks, &cnt, &r, nullptr);
        if (rc) return rc;
        st.large_calls++;
        st.rows_verified += n + 1;
        if (r < n) {
            st.rollbacks++;
            st.tokens_discarded += n - r;
        }
        last = toks[r];
    }
    st.n_generated = s->y_len - s->n0;
    *n_out = st.n_generated;
    if (st.n_generated > 0) {
        HIPC(hipMemcpyAsync(out, s->y + s->n0, sizeof(int) * (size_t)st.n_generated, hipMemcpyDeviceToHost,
                            s->stream));
        HIPC(hipStreamSynchronize(s->stream));
    }
    if (stats) *stats = st;
    return BILD_OK;
}

extern "C" int bild_greedy(bild_state* s, int which, const int32_t* src, int n_src, int max_new, int32_t eos,
                           int32_t* out, int32_t* n_out) {
    if (!s || !out || !n_out || max_new < 0 || which < 1 || which > 2) return BILD_EINVAL;
    int rc = BILD_OK;
    if (src) {
        rc = bild_encode(s, src, n_src);
        if (rc) return rc;
    } else if (!s->encoded) {
        return BILD_ESTATE;
    }
    if (s->n0 + max_new > s->max_len) return BILD_ECAP;
    const int w = which - 1;
    int last = -1;
    while (s->y_len - s->n0 < max_new && !(s->y_len > s->n0 && last == eos && eos >= 0)) {
        rc = catch_up(s, w, s->y_len - 1);
        if (rc) return rc;
        rc = run_pass(s, w, 1, 1, 2);
        if (rc) return rc;
        rc = pull_ctl(s);
        if (rc) return rc;
        last = s->hctl->res_tok;
    }
    // leave the state consistent for a following BiLD call: the other model lags, which is allowed
    *n_out = s->y_len - s->n0;
    if (*n_out > 0) {
        HIPC(hipMemcpyAsync(out, s->y + s->n0, sizeof(int) * (size_t)*n_out, hipMemcpyDeviceToHost, s->stream));
        HIPC(hipStreamSynchronize(s->stream));
    }
    return BILD_OK;
}

namespace {
int alloc_logit_buffers(bild_state* s) {
    for (int w = 0; w < 2; ++w) {
        if (s->ms[w].dbg) continue;
        int rc = dev_alloc(s->allocs, (void**)&s->ms[w].dbg, sizeof(float) * kMaxRows * (size_t)s->ms[w].m->cfg.vocab);
        if (rc) return rc;
    }
    return BILD_OK;
}
}  // namespace

extern "C" int bild_debug_enable_logits(bild_state* s, int enable) {
    if (!s) return BILD_EINVAL;
    if (enable) {
        int rc = alloc_logit_buffers(s);
        if (rc) return rc;
    }
    s->debug_logits = enable != 0;
    return BILD_OK;
}

extern "C" int bild_set_sampling(bild_state* s, float top_p, const float* u_small, const float* u_large, int n) {
    if (!s) return BILD_EINVAL;
    // captured passes carry top_p by value: a new value starts from fresh captures
    auto drop_graphs = [&]() {
        (void)hipStreamSynchronize(s->stream);
        for (auto& kv : s->graphs) (void)hipGraphExecDestroy(kv.second);
        s->graphs.clear();
    };
    if (!(top_p > 0.f)) {  // back to argmax (and to the threshold rule of the review, which is all argmax decoding has)
        if (s->top_p > 0.f) drop_graphs();
        s->top_p = 0.f;
        s->accept_mode = 0;
        return BILD_OK;
    }
    if (top_p > 1.f || !u_small || !u_large || n < s->max_len) return BILD_EINVAL;
    const float* us[2] = {u_small, u_large};
    for (int w = 0; w < 2; ++w)
        for (int i = 0; i < s->max_len; ++i)
            if (!(us[w][i] >= 0.f && us[w][i] < 1.f)) return BILD_EINVAL;
    int rc = alloc_logit_buffers(s);
    if (rc) return rc;
    HIPC(hipStreamSynchronize(s->stream));
    for (int w = 0; w < 2; ++w) {
        if (!s->u_dev[w]) {
            rc = dev_alloc(s->allocs, (void**)&s->u_dev[w], sizeof(float) * (size_t)(s->max_len + 1));
            if (rc) return rc;
        }
        HIPC(hipMemcpy(s->u_dev[w], us[w], sizeof(float) * (size_t)s->max_len, hipMemcpyHostToDevice));
    }
    if (!s->draw_ws) {
        rc = dev_alloc(s->allocs, (void**)&s->draw_ws, sizeof(DrawWs));
        if (rc) return rc;
        HIPC(hipMemset(s->draw_ws, 0, sizeof(DrawWs)));
        drop_graphs();  // (none can have been captured with a draw yet; kept for safety)
    }
    if (s->top_p != top_p) drop_graphs();
    s->top_p = top_p;
    return BILD_OK;
}

extern "C" int bild_set_acceptance(bild_state* s, int rule, const float* u_accept, int n) {
    if (!s || (rule != BILD_ACCEPT_THRESHOLD && rule != BILD_ACCEPT_REJECTION)) return BILD_EINVAL;
    auto drop_graphs = [&]() {  // captured passes carry the rule by value
        (void)hipStreamSynchronize(s->stream);
        for (auto& kv : s->graphs) (void)hipGraphExecDestroy(kv.second);
        s->graphs.clear();
    };
    if (rule == BILD_ACCEPT_THRESHOLD) {
        if (s->accept_mode != 0) drop_graphs();
        s->accept_mode = 0;
        return BILD_OK;
    }
    if (!(s->top_p > 0.f)) return BILD_ESTATE;
    if (!u_accept || n < s->max_len) return BILD_EINVAL;
    for (int i = 0; i < s->max_len; ++i)
        if (!(u_accept[i] >= 0.f && u_accept[i] < 1.f)) return BILD_EINVAL;
    HIPC(hipStreamSynchronize(s->stream));
    if (!s->u_acc) {
        const size_t V = (size_t)s->pair->m[0]->cfg.vocab;
        int rc = dev_alloc(s->allocs, (void**)&s->u_acc, sizeof(float) * (size_t)(s->max_len + 1));
        if (rc) return rc;
        rc = dev_alloc(s->allocs, (void**)&s->s_ring, sizeof(float) * (size_t)kMaxRows * V);
        if (rc) return rc;
        rc = dev_alloc(s->allocs, (void**)&s->s_draw, sizeof(float4) * (size_t)(s->max_len + 1));
        if (rc) return rc;
        HIPC(hipMemset(s->s_ring, 0, sizeof(float) * (size_t)kMaxRows * V));
        HIPC(hipMemset(s->s_draw, 0, sizeof(float4) * (size_t)(s->max_len + 1)));
    }
    HIPC(hipMemcpy(s->u_acc, u_accept, sizeof(float) * (size_t)s->max_len, hipMemcpyHostToDevice));
    if (s->accept_mode != 1) drop_graphs();
    s->accept_mode = 1;
    return BILD_OK;
}

extern "C" int bild_debug_logits(bild_state* s, int which, int row, float* out) {
    if (!s || !out || which < 1 || which > 2) return BILD_EINVAL;
    ModelState& M = s->ms[which - 1];
    if (!s->debug_logits || !M.dbg) return BILD_ESTATE;
    if (row < 0 || row >= M.last_rows) return BILD_EINVAL;
    const size_t V = M.m->cfg.vocab;
    HIPC(hipMemcpyAsync(out, M.dbg + (size_t)row * V, sizeof(float) * V, hipMemcpyDeviceToHost, s->stream));
    HIPC(hipStreamSynchronize(s->stream));
    return BILD_OK;
}

extern "C" int bild_debug_kv(bild_state* s, int which, int layer, int is_v, int pos0, int n, float* out) {
    if (!s || !out || which < 1 || which > 2 || n < 1 || pos0 < 0) return BILD_EINVAL;
    if (!s->encoded) return BILD_ESTATE;
    const ModelState& M = s->ms[which - 1];
    const bild_model* m = M.m;
    // an early-exit pair keeps the trunk's rows in the large model's buffers: the view has its own layer count
    if (layer < 0 || layer >= m->cfg.n_dec_layers || pos0 + n > s->len[which - 1]) return BILD_EINVAL;
    const size_t I = m->inner(), esz = m->esz(), cap = s->cap_len;
    std::vector<char> raw((size_t)(is_v ? I * cap : (size_t)n * I) * esz);
    const char* base = (is_v ? M.vcache : M.kcache) + (size_t)layer * cap * I * esz;
    HIPC(hipStreamSynchronize(s->stream));
    // K is [position][I]; V is stored transposed, [I][capacity]
    HIPC(hipMemcpy(raw.data(), is_v ? base : base + (size_t)pos0 * I * esz, raw.size(), hipMemcpyDeviceToHost));
    auto widen = [&](size_t idx) -> float {
        if (esz == 4) return ((const float*)raw.data())[idx];
        const uint32_t u = (uint32_t)((const uint16_t*)raw.data())[idx] << 16;
        float f;
        std::memcpy(&f, &u, 4);
        return f;
    };
    for (int t = 0; t < n; ++t)
        for (size_t i = 0; i < I; ++i) out[(size_t)t * I + i] = is_v ? widen(i * cap + pos0 + t) : widen((size_t)t * I + i);
    return BILD_OK;
}

extern "C" const char* bild_strerror(int code) {
    switch (code) {
        case BILD_OK: return "ok";
        case BILD_EINVAL: return "invalid argument";
        case BILD_ESTATE: return "call not valid in the current state";
        case BILD_ECAP: return "capacity exceeded";
        case BILD_EHIP: return "HIP runtime error";
        case BILD_ENOMEM: return "out of memory";
        default: return "unknown error";
    }
}
