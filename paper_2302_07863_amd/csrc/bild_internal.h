// Internal structures shared by the host runtime and the HIP kernels of the
// BiLD library (gfx950).  Not part of the public ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bild.h"

namespace bild {

constexpr int kMaxRows = BILD_MAX_ROWS;  // rows per decoder pass
constexpr int kTileBytes = 1024;         // one streamed weight tile: 16 output features x KT inputs

// A weight matrix in streaming layout.  Logical shape [n features][k inputs]
// (y = W x).  It is cut into tiles of 16 features x KT inputs (KT = 32 for bf16,
// 16 for fp32), each 1 KiB and stored in the register order of the matrix-core
// A operand: lane l of a wavefront owns the 16 bytes at l*16, which hold feature
// (l % 16) and inputs (l / 16) * KT/4 .. +KT/4-1 of the tile.  Tiles of one
// feature block are contiguous along k, so a wavefront streaming along k issues
// back-to-back 1 KiB coalesced loads.  Features beyond n are zero padding.
struct TMat {
    const void* w = nullptr;
    int n = 0;   // features (rows of the logical matrix)
    int k = 0;   // inputs
    int tn = 0;  // feature tiles = ceil(n / 16)
    int tk = 0;  // input tiles   = k / KT
};

// Device-resident control block of one request.  Kernels read lengths from here
// so that a captured launch sequence stays valid as the sequence grows.
struct Ctl {
    int y_len;
    int draft_start;
    int len[2];       // consumed rows per model: [0] small, [1] large
    int n_src;        // source length (cross-attention keys) or prompt length
    int n_max;
    float alpha_fb;   // thresholds of the two policies (Sections 3.3, 3.4), read by the policy kernel
    float alpha_rb;
    // results of the last pass, mirrored to the host after it
    int res_tok;
    int res_flag;
    int res_r;
    int res_n;
    float res_pmax;
    int pad0;
    float res_nll[kMaxRows];
    int res_rowtok[kMaxRows];  // argmax of every row of the last pass
    int seq;          // passes finished so far; the LAST word, and the last one the policy kernel mirrors to the host
};

// Partial softmax statistics of one row over a slice of the vocabulary.
struct StatPart {
    float m;    // max logit
    float s;    // sum exp(z - m)
    int idx;    // argmax (lowest id among equal maxima)
    int pad;
};

enum Epilogue : int {
    EPI_STORE = 0,  // out[t][n] = v
    EPI_RESID = 1,  // out[t][n] += v
    EPI_QKV = 2,    // n < q_dim -> q_out; then K rows, then V rows of the cache (RoPE on q, k)
    EPI_ACT = 3,    // out[t][n] = act(v) or act(gate) * up for gated FFNs
    EPI_LMHEAD = 4, // z = scale * v; softmax partials, logit of the target token
    EPI_PART = 5    // out[slice][t][n] = v over a slice of the inputs, no norm (see GemmArgs::ksplit)
};

struct GemmArgs {
    TMat W;
    const float* x;  // [T][ldx] fp32 activations
    int ldx;
    int T;
    const float* gain;  // non-null: RMSNorm prologue, x_hat = x * rsqrt(mean x^2 + eps) * gain
    float eps;
    int epi;
    float* out;
    int ldo;
    // EPI_QKV
    int q_dim;      // features [0, q_dim) are queries (0 for a K/V-only projection)
    int i_dim;      // inner dim I; K features follow q, V features follow K
    float* q_out;   // [T][I] fp32
    void* k_cache;  // [capacity][I] in the model dtype
    void* v_cache;  // transposed: [I][vcap], position contiguous
    int vcap;
    const int* pos_ptr;  // position of row 0 = (pos_ptr ? *pos_ptr : 0) + pos_add
    int pos_add;
    int rope;
    float rope_base;
    int d_head;
    // EPI_ACT
    int act;
    // EPI_LMHEAD
    float scale;
    int vocab;
    const int* y;        // sequence; target of row t is y[*pos_ptr + pos_add + t + 1] if below *ylen_ptr
    const int* ylen_ptr;
    StatPart* part;      // [gridDim.x][kMaxRows]
    float* zt;           // [kMaxRows] logit of each row's target
    float* dbg;          // nullable [T][vocab] full logits (tests only)
    int row_off;         // row index of x row 0 within the pass (for part / zt / dbg / targets)
    // x given as key-split attention partials (mg_splits > 1): x[t][n] = sum_s w_s O_s[t][n] / sum_s w_s L_s,
    // w_s = exp(m_s - max_s m_s), with (m_s, L_s) per (row, head n / d_head); the GEMM merges them while staging
    int mg_splits;
    const float* mg_o;   // [mg_splits][T][ldx] unnormalised outputs
    const float* mg_ml;  // [mg_splits][T][mg_heads][2]
    int mg_heads;
    // A projection with few output features and many inputs may be cut into `ksplit` slices of its inputs, each slice a
    // workgroup row of its own (blockIdx.y) that writes out + slice * part_stride (EPI_PART); its reader then takes
    // x = base + sum of the slices (px, pn = ksplit) while staging and writes the sum to x_out.
    int ksplit;             // > 1: EPI_PART launch over blockIdx.y slices; W.tk must be a multiple of it
    int64_t part_stride;    // floats between the outputs of consecutive slices
    int k_len;              // (set by the launch wrapper) inputs of this workgroup's slice
    int k_off_tiles;        // (set by the launch wrapper) first input tile of the slice
    const float* px;        // reader: pn partial results [pn][px_stride] laid out like x
    int64_t px_stride;
    int pn;                 // 0 or kPartSlices
    float* x_out;           // reader: where workgroup 0 writes base + partial results ([T][ldx], not x itself)
    // bf16 models, passes of a few rows: activations travel between projections as two bf16 planes (high part and
    // low part of each value, [T][ld]) written once by the producer, with the consumer's norm gain already applied
    const uint16_t* xb_hi;  // input planes (non-null: x, gain are not read; ldx is their row stride)
    const uint16_t* xb_lo;
    const float* ssq_part;  // [ssq_parts][kMaxRows]: partial sums of x^2 per row, one per producer wave (norm only)
    int ssq_parts;
    uint16_t* nx_hi;        // output planes for the next projection (EPI_RESID: of out * nx_gain, beside the fp32 out;
    uint16_t* nx_lo;        //  EPI_ACT: of the activation, instead of the fp32 out)
    const float* nx_gain;   // EPI_RESID: gain of the norm in front of the next projection
    float* nx_ssq;          // EPI_RESID: [feature tiles / rw][kMaxRows] sums of out^2 per owner wave
    int nx_ld;
    // Single-row passes: the first projection of the pass may gather its input row from the embedding matrix itself
    // (e_w non-null; x is not read): x = e_scale * E[(tokens[base] + e_shift) mod e_vocab] (+ e_pe[base], the position
    // table, if non-null) with base = *e_base_ptr + e_base_add; workgroup 0 also writes the row to x_out.
    const void* e_w;        // tiles of the embedding matrix
    int e_tk;               // its input tiles per feature block
    const int* e_tokens;
    const int* e_base_ptr;
    int e_base_add;
    int e_vocab;
    int e_shift;            // 0 <= e_shift < e_vocab
    float e_scale;
    const float* e_pe;      // nullable: [positions][k]
    // launch shape
    int wk;   // input slices per workgroup (a power of two)
    int lwk;  // (set by the kernel) log2(wk)
    int nwv;  // waves per workgroup = wk * feature groups (4 or 8)
    int rw;   // feature tiles per wave (1, or 2 for gated FFNs)
    int kc;   // inputs staged in LDS per chunk
};

// The leading scalar arguments of the GEMM kernels (gemm_body.h, BILD_GEMM_HOT_PARAMS), from a filled GemmArgs.
static inline int gemm_hot_geom(const GemmArgs& a) {
    int lwk = 0;
    while ((1 << lwk) < a.wk) ++lwk;
    return a.wk | (lwk << 4) | (a.nwv << 8) | (a.T << 12);
}
#define BILD_GEMM_HOT_MID(a) (a).W.tn, (a).W.tk, gemm_hot_geom(a), (a).kc, (a).ldx
#define BILD_GEMM_HOT(a) (a).W.w, (const void*)(a).x, (const void*)(a).gain, (a).px, BILD_GEMM_HOT_MID(a), ((a).x_out ? (int)((a).x_out - (a).x) : 0)
#define BILD_GEMM_HOT_PRE(a) (a).W.w, (const void*)(a).xb_hi, (const void*)(a).xb_lo, (a).px, BILD_GEMM_HOT_MID(a), 0
#define BILD_GEMM_HOT_MG(a) (a).W.w, (const void*)(a).mg_o, (const void*)(a).mg_ml, (a).px, BILD_GEMM_HOT_MID(a), ((a).mg_heads | ((a).d_head << 16))

struct AttnArgs {
    const float* q;  // [T][I]
    const void* k;   // [capacity][I]
    const void* v;   // transposed: [I][vcap]
    int vcap;
    int nw;          // waves per workgroup
    float* out;      // [T][I]
    int T, heads, d_head, i_dim;
    int causal;                // 1: row t sees keys <= base + t
    const int* len_ptr;        // never null.  causal: base = *len_ptr + base_add = position of row 0;
    int base_add;              // non-causal: number of keys = nkeys_fixed if > 0, else *len_ptr
    int nkeys_fixed;
    int splits;                // key ranges handled by separate workgroups
    int lsplits;               // (set by the kernel) log2(splits): splits is a power of two
    int defer_merge;           // splits > 1: leave the partials for the consumer GEMM to merge (no merge kernel)
    float* part_o;             // [splits][T][I]   unnormalised partial outputs
    float* part_ml;            // [splits][T][heads][2] (max, sum)
    float scale;
    // relative-position models: score(row, key) += rel_bias[head][clamp(key_pos - row_pos, -rel_d, rel_d) + rel_d];
    // row_pos = base + t (causal) or base_add + t (not causal).  Null: no bias.
    const float* rel_bias;      // [heads][2*rel_d + 1]
    int rel_d;
    // non-null (bf16 models): the finished output goes to these bf16 planes [T][I] (high and low part of each value,
    // what the output projection stages) instead of `out`; not used while the partials are left to the consumer
    uint16_t* ob_hi;
    uint16_t* ob_lo;
    // attention fused with the output projection (launch_attention_proj): W_o, the partial results of the residual
    // update, one per head ([heads][proj_stride], laid out [T][d_model]), and the number of column groups
    TMat wo;
    float* proj_out;
    int64_t proj_stride;
    int cgroups;
    int d_model;
};

struct EmbedArgs {
    TMat E;
    const int* tokens;      // token of row t is tokens[base + t]
    const int* base_ptr;    // base = (base_ptr ? *base_ptr : 0) + base_add; also the position of row 0
    int base_add;
    int T, d, vocab, tie_shift, sinusoidal;
    float embed_scale;
    float* x;  // [T][d]
    const float* pe;  // nullable: sinusoidal position table [positions][d] (launch_pe_table), read instead of evaluating sin / cos
    // non-null (bf16 models): x * nx_gain also as bf16 planes [T][d] for the first projection, and the sum of x^2 of
    // each row in four parts (one per wave), nx_ssq[wave][kMaxRows]
    uint16_t* nx_hi;
    uint16_t* nx_lo;
    const float* nx_gain;
    float* nx_ssq;
};
constexpr int kEmbedSsqParts = 4;
constexpr int kPartSlices = 4;      // input slices of a split projection (EPI_PART) = partial results its reader adds
constexpr int kMaxSsqParts = 256;  // partial sums of squares a consumer adds per row

// Copies T rows of d floats: dst[dst_row + t] = src[src_row + t], each row index = (*ptr or 0) + add.
// Carries the hidden state between the shared trunk and the upper layers of an early-exit pair.
struct RowCopyArgs {
    const float* src;
    float* dst;
    const int* src_row_ptr;
    const int* dst_row_ptr;
    int src_row_add, dst_row_add;
    int d, T;
};

struct FinishArgs {
    Ctl* ctl;
    int* y;
    const StatPart* part;
    int nparts;
    const float* zt;
    int T;       // rows that went through the LM head
    int row_off; // first such row within the pass
    int which;   // 0 small, 1 large
    int mode;    // 0 small step, 1 verify, 2 plain greedy (always append), 3 advance only, 4 measure
    int rows_consumed;  // rows the pass consumed (cache advance)
    int y_cap;
    Ctl* host_mirror;   // device-visible pinned host copy of the control block, written last
    // sampling variant (top_p > 0): the committed token is drawn from the nucleus of its row instead of the argmax
    float top_p;
    const float* logits;  // [rows][vocab] logits of the pass (row_off applies)
    int vocab;
    const float* u;       // uniform number per sequence position, for the model of this pass
    // rejection-sampling acceptance (accept_mode 1, sampling variant only): the review keeps a draft iff
    // u_acc[position] * p_S(draft) < p_L(draft) and replaces the first refused one by a draw from max(0, p_L - p_S)
    int accept_mode;
    const float* u_acc;   // uniform number per sequence position for the acceptance test
    float* s_ring;        // [kMaxRows][vocab] the small model's logits of each pending draft, by draft index
    float4* s_draw;       // [sequence capacity] (max logit, nucleus threshold key, nucleus mass, -) of the small model's row
    // nucleus draw spread over the chip (launch_finish_draw): its workspace
    struct DrawWs* dws;
};

// Workspace of the nucleus draw that is spread over many workgroups (policy.hip).  Probability masses are integers
// there: exp(z - max) in units of 2^-40, so sums do not depend on the order of their terms and atomics stay reproducible.
constexpr int kDrawSliceIds = 1024;   // ids per workgroup of a sweep
constexpr int kDrawMaxSlices = 1024;  // vocabularies of up to 1 048 576 ids
struct DrawWs {
    int row, pos;                     // row of the pass the token is drawn from, sequence position it will take
    float m;                          // that row's largest logit
    uint32_t key;                     // nucleus threshold: members have float_key(z) >= key
    unsigned long long mass;          // mass of the nucleus
    unsigned long long pad;
    StatPart merged[kMaxRows];        // merged LM-head statistics of the pass (one "partial" per row for the commit)
    unsigned long long hist[4][256];  // mass per value of key byte 3 (most significant) .. 0 among the keys still in play
    unsigned long long slice[kDrawMaxSlices];  // members' mass per slice of kDrawSliceIds ids
};

size_t gemm_lds_bytes(const GemmArgs& a, int dtype);

// launch wrappers (kernels.hip); each returns the hipError_t of the launch
hipError_t launch_gemm(const GemmArgs& a, int dtype, hipStream_t st);
// kDenseMinRows rows or more: the dense-tile kernel (gemm_dense.hip); launch_gemm forwards to it
constexpr int kDenseMinRows = 513;
constexpr int kDenseRows = 64;   // rows per workgroup
constexpr int kDenseWaves = 4;
constexpr int kDenseRW = 4;      // feature tiles per wave
constexpr int dense_kc(int) { return 128; }  // inputs staged per chunk
size_t dense_lds_bytes(int dt);
hipError_t launch_gemm_dense(const GemmArgs& a, int dtype, hipStream_t st);
// bf16 passes whose activations travel as planes (gemm_pre.hip); launch_gemm forwards to it
hipError_t launch_gemm_pre(const GemmArgs& a, hipStream_t st);
hipError_t gemm_pre_init();
hipError_t launch_attention(const AttnArgs& a, int dtype, hipStream_t st);
hipError_t launch_attention_proj(const AttnArgs& a, int dtype, hipStream_t st);
constexpr int kMaxHeadParts = 16;   // heads whose partial results one reader adds (attention fused with its output projection)
hipError_t launch_embed(const EmbedArgs& a, int dtype, hipStream_t st);
// table[pos][k] = sin / cos of pos * 10000^(-2 floor(k/2) / d) (k even / odd), evaluated in double precision as embed_kernel does
hipError_t launch_pe_table(float* table, int positions, int d, hipStream_t st);
hipError_t launch_finish(const FinishArgs& a, hipStream_t st);
// sampling variant with the threshold rule: the same result as launch_finish, the draw spread over the chip (seven launches)
hipError_t launch_finish_draw(const FinishArgs& a, hipStream_t st);
constexpr int kFinishDrawStages = 7;
hipError_t launch_row_copy(const RowCopyArgs& a, hipStream_t st);
hipError_t kernels_init();  // one-time function attributes; call before any stream capture
hipError_t attention_init();  // (attention.hip; called by kernels_init)
size_t gemm_num_blocks(const GemmArgs& a);
size_t attn_lds_bytes(int dtype, int d_head, int T, int nw);
void gemm_pick_shape(GemmArgs& a, int dtype);

// host-side re-layout (layout.cpp)
// src is [k][n] row-major (math layout, y = x W) when transposed_src, else [n][k].
void tile_matrix(const float* src, bool src_is_k_by_n, int n, int k, int dtype, void* dst);
size_t tiled_bytes(int n, int k, int dtype);
// interleave gate/up feature tiles of a gated FFN: dst tiles 2j = gate tile j, 2j+1 = up tile j
void tile_gated_pair(const float* gate_k_by_n, const float* up_k_by_n, int n, int k, int dtype, void* dst);
// concatenate several [k][n_i] matrices along the feature axis
void tile_concat(const float* const* srcs, const int* ns, int count, int k, int dtype, void* dst);

}  // namespace bild
