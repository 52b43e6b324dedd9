// Host-side objects behind the opaque handles of bild.h, shared by the product entry points (bild_api.hip)
// and the measurement entry points (bench_api.hip).  Not part of the public ABI.
#pragma once
#include <array>
#include <map>
#include <vector>

#include "bild_internal.h"

#define HIPC(expr)                                   \
    do {                                             \
        hipError_t e_ = (expr);                      \
        if (e_ != hipSuccess) return BILD_EHIP;      \
    } while (0)

using bild::Ctl;
using bild::StatPart;
using bild::TMat;
using bild::kMaxRows;

struct LayerW {
    const float* ln1 = nullptr;
    TMat wqkv, wo;
    const float* lnc = nullptr;
    TMat cwq, cwkv, cwo;
    const float* ln2 = nullptr;
    TMat win, wout;
};

struct bild_model {
    bild_model_config cfg;
    TMat emb, head;
    const float* enc_final = nullptr;
    const float* dec_final = nullptr;
    const float* enc_rel = nullptr;  // relative-position models: [heads][2*rel_max_dist + 1] score biases of the
    const float* dec_rel = nullptr;  // encoder's / decoder's self-attention, shared by all layers of the stack
    std::vector<LayerW> enc, dec;
    std::vector<void*> allocs;
    size_t device_bytes = 0;
    int inner() const { return cfg.n_heads * cfg.d_head; }
    int esz() const { return cfg.dtype == BILD_DT_BF16 ? 2 : 4; }
    bool gated() const { return cfg.act != BILD_ACT_RELU; }
    size_t layer_weight_bytes() const {  // weight matrices of one decoder layer
        const size_t d = cfg.d_model, I = inner(), F = cfg.d_ff;
        return (4 * d * I * (cfg.cross_attn ? 2 : 1) + (gated() ? 3 : 2) * d * F) * esz();
    }
};

struct bild_pair {
    bild_model* m[2];  // [0] small, [1] large
    bool decoder_only;
    bool small_borrows_encoder;
    int trunk_layers = 0;        // > 0: early-exit pair, m[0] is a view of m[1]'s first trunk_layers decoder layers
    bild_model* view = nullptr;  // that view (owned by the pair; it owns no device memory)
};

struct ModelState {
    const bild_model* m = nullptr;
    char* kcache = nullptr;  // [L][cap][I]
    char* vcache = nullptr;
    char* ck = nullptr;      // cross [L][max_src][I]
    char* cv = nullptr;
    float *x = nullptr, *q = nullptr, *a = nullptr, *h = nullptr;  // [rows_cap][d], [rows_cap][I], [rows_cap][I], [rows_cap][F]
    int rows_cap = kMaxRows;  // rows one decoder pass may carry (the whole prompt for decoder-only prefill)
    StatPart* part = nullptr;
    int nparts_cap = 0;
    float* zt = nullptr;
    float* dbg = nullptr;     // [32][vocab], only when debugging
    float* att_o = nullptr;   // split-key partials
    float* att_ml = nullptr;
    int max_splits = 1;
    // encoder scratch (models with an encoder)
    float* enc_x = nullptr;   // [max_src][d]
    float* enc_q = nullptr;   // [max_src][I]
    float* enc_a = nullptr;   // [max_src][I]
    float* enc_h = nullptr;   // [max_src][F]
    char* enc_k = nullptr;    // [max_src][I]
    char* enc_v = nullptr;
    int last_rows = 0;        // rows of the last LM-head pass (for debug logits)
    // bf16 models: activations of a pass of a few rows as high / low bf16 planes (see GemmArgs::xb_hi)
    uint16_t* xb = nullptr;   // [2][32][d]   residual stream times the next norm's gain
    uint16_t* ab = nullptr;   // [2][32][I]   attention output
    uint16_t* hb = nullptr;   // [2][32][F]   FFN hidden
    float* ssq = nullptr;     // [d / 16 + 8][32] partial sums of squares beside xb
    float* x2 = nullptr;      // [32][d] second residual-stream buffer (see GemmArgs::x_out)
    float* px = nullptr;      // [kPartSlices][32][d] partial results of a split FFN output projection
    float* pxh = nullptr;     // [kMaxHeadParts][32][d] one partial result per head of attention fused with its output projection
    float* pe = nullptr;      // sinusoidal models: position table [cap_len][d] for the decoder's embedding
};

struct bild_state {
    const bild_pair* pair = nullptr;
    ModelState ms[2];
    Ctl* ctl = nullptr;   // device
    Ctl* hctl = nullptr;  // pinned host mirror of the control block, written by the policy kernel
    int seq_issued = 0;   // passes with a policy kernel enqueued so far (the device counts them in Ctl::seq)
    Ctl* hctl_dev = nullptr;  // the same buffer as the device sees it
    float* halpha = nullptr;  // pinned staging for threshold updates
    float alpha_fb = -1.f, alpha_rb = -1.f;  // thresholds currently in the device control block
    bool use_graphs = true;
    int ksplit_max_d = 2048;      // ... of models up to this wide (7B-shaped small model, 2048 wide: 0.729 -> 0.717 ms per step)
    int ksplit_min_f = 2048;      // FFN widths from which the output projection of a narrow model (d <= 1024) is cut into input slices
    int fuse_max_kv = 32 << 10;   // ... while one head's cached K/V are at most this many bytes
    bool fuse_attn = true;        // single-row passes of narrow models: attention and its output projection in one kernel
    bool fuse_embed = true;       // single-row passes: the first projection gathers its input row from the embedding matrix
    int pre_min_rows = 0;         // > 0 (experiments): row count from which a bf16 pass hands activations on as bf16 planes
    bool gemm_only = false;       // measurement: a pass launches only its weight-streaming GEMMs
    int64_t gemm_count = 0, gemm_bytes = 0;  // tallied while a pass is being issued
    int stage_count = 0;          // kernel launches of the pass issued last (counted also where a measurement skips the launch)
    std::map<std::array<int, 6>, hipGraphExec_t> graphs;  // captured passes by (model, rows, lm rows, mode, key bucket, debug)
    float top_p = 0.f;         // > 0: sampling variant, tokens are drawn from the nucleus
    float* u_dev[2] = {nullptr, nullptr};  // uniform number per sequence position, per model
    bild::DrawWs* draw_ws = nullptr; // workspace of the draw that is spread over the chip
    bool draw_spread = true;   // false (BILD_DRAW_ONE_WG=1, tests): every draw by the single workgroup of the policy kernel
    int accept_mode = 0;       // 1: the review uses the rejection-sampling rule (needs top_p > 0)
    float* u_acc = nullptr;    // uniform number per sequence position for that rule
    float* s_ring = nullptr;   // [kMaxRows][vocab] the small model's logits of the pending drafts
    float4* s_draw = nullptr;  // [max_len + 1] (max, threshold key, nucleus mass) of the small model's row per position
    float* trunk_x = nullptr;  // early-exit pair: [cap_len][d] hidden state after the trunk's last layer, by position
    int* y = nullptr;     // device [max_len + 1]
    int* src = nullptr;   // device [max_src]
    hipStream_t stream = nullptr;
    bool own_stream = false;
    int max_src = 0, max_len = 0, n_max = 0;
    int cap_len = 0, cap_src = 0;  // cache capacities: max_len / max_src rounded up to 32 rows
    // host mirror of the control block (kept exact by reading back after every pass)
    int y_len = 0, draft_start = 0, len[2] = {0, 0}, n_src = 0, n0 = 0;
    bool encoded = false;
    bool debug_logits = false;
    std::vector<void*> allocs;
    std::vector<void*> host_allocs;
    // event bracketing of GEMM launches (measurement only)
    bool prof_on = false;
    int prof_cap = 0, prof_used = 0, prof_dropped = 0;
    std::vector<hipEvent_t> prof_ev;
    struct ProfRec { int model, cls; int64_t bytes; };
    std::vector<ProfRec> prof_rec;
};


namespace bild {
// shared host logic (bild_api.hip)
int dev_alloc(std::vector<void*>& keep, void** p, size_t bytes);
int key_bucket(int nkeys);
int catch_up(bild_state* s, int w, int target);
int run_pass(bild_state* s, int w, int T, int lm_rows, int mode);
int decoder_pass(bild_state* s, int w, int T, int lm_rows, int mode, int key_hint);
int pick_splits_raw(int d_head, int esz, int max_splits, int nkeys, int heads, int T, bool* defer);
int pick_attn_waves(int dtype, int d_head, int T, int nkeys, int splits);
}  // namespace bild
