// HIP kernels of the BiLD decoding path for gfx950 (CDNA4, wave64).
//
//   gemm_body        weight-streaming skinny GEMM  y[T][N] = f(x[T][K]) W^T for T <= 32 rows
//                    (T = 1: the small model's autoregressive step; T = n+1: the large
//                    model's non-autoregressive review, Section 3.2), with the RMSNorm of
//                    the input fused in front and the consumer (K/V cache append + RoPE,
//                    activation, residual add, LM-head softmax statistics) fused behind.
//                    Launched as gemm_kernel (any T <= 32), gemm_row_kernel (T = 1 at compile
//                    time), gemm_few_kernel (2-4 rows), gemm_merge_kernel (input still in key-split
//                    attention partials) and gemm_rows_kernel (an encoder over up to a few hundred rows: blocks of
//                    32 rows).  Longer passes (prompt prefill) go to the dense-tile kernel of gemm_dense.hip.
//   attn_body        KV-cache attention for T query rows of one head (attn_kernel; attn_rows_kernel
//                    for more than 32 query rows; attn_merge_kernel joins key splits).
//   embed_kernel     embedding gather + sinusoidal position.
// (The policy kernels - merge of the LM-head statistics, fallback / rollback tests, commit, draws - are in policy.hip.)
//
// The path is bound by memory: every weight byte is read once per pass and the arithmetic
// per byte is tiny - by HBM bandwidth where the matrices are large (7B-class widths), by the
// latency of each stage's first cold access where they are small (T5-class).  Weights sit in HBM in the exact register order
// of the matrix-core A operand (see bild::TMat) so that one wavefront load instruction
// moves 1 KiB of contiguous memory straight into MFMA operand registers; activations
// (a few KiB) are staged once per workgroup in LDS as the B operand.  bf16 models keep
// activations at fp32 accuracy by splitting each value into a high and a low bf16 part
// and issuing two MFMAs per weight tile; the matrix cores have an order of magnitude
// more throughput than the stream needs, so this is free.
#include "kernel_common.h"
#include "gemm_body.h"

namespace bild {


// SHORT: no wave has more than one batch of tiles - the second weight buffer does not exist (see gemm_row_kernel).
template <int DT, int RW, int EPI, int ROPE, int NT, bool SHORT = false>
__global__ __launch_bounds__(512) void gemm_kernel(BILD_GEMM_HOT_PARAMS, const GemmArgs a0) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const GemmArgs a = gemm_hot<HOT_X, DT>(a0, BILD_GEMM_HOT_NAMES);
    gemm_body<DT, RW, EPI, ROPE, NT, gemm_batch(RW, false, NT), 0, false, !SHORT>(a, (int)blockIdx.x, smem);
}

// The single-row pass (the small model's step, the large model's plain step): the row count is a
// compile-time 1, which removes the multi-row staging paths from the code.
// Padding tiles are not free: a batch slot past the wave's range still costs a load of a clamped tile and, in the
// first buffer, two MFMAs, and on the latency-bound shapes that is most of a wave's instructions (measured on the T5
// pair: 236 -> 206 us per small-model step and 1048 -> 962 us per large-model step once the 512- and 1024-wide inputs
// stopped padding 8 tiles per wave to 24).  VAR picks the batch geometry by the tiles a wave has:
//   1: at most 8   - one batch of 8, no second buffer
//   3: exactly 8 in every wave (RW = 1) - the same without clamped tile indices (gemm_body, EX)
//   2: at most 16  - two batches of 8
//   0: more        - batches of 12 (more bytes in flight for the bandwidth-bound shapes)
constexpr int kShortBatch = 8;
template <int DT, int RW, int EPI, int ROPE, int VAR = 0, int PS = 0>
__global__ __launch_bounds__(512) void gemm_row_kernel(BILD_GEMM_HOT_PARAMS, const GemmArgs a0) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const GemmArgs a = gemm_hot<HOT_X, DT>(a0, BILD_GEMM_HOT_NAMES);
    gemm_body<DT, RW, EPI, ROPE, 1, VAR ? kShortBatch / RW : gemm_batch(RW, true), 0, true, VAR != 1 && VAR != 3, 0, false, false, PS, false,
              false, VAR == 3>(a, (int)blockIdx.x, smem);
}

// The first projection of a single-row pass, gathering its input row from the embedding matrix (gemm_body, EMB): the
// pass then has no embedding kernel, one dependent stage fewer.
template <int DT, int ROPE, int VAR>
__global__ __launch_bounds__(512) void gemm_row_embed_kernel(BILD_GEMM_HOT_PARAMS, const GemmArgs a0) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const GemmArgs a = gemm_hot<HOT_X, DT>(a0, BILD_GEMM_HOT_NAMES);
    gemm_body<DT, 1, EPI_QKV, ROPE, 1, VAR ? kShortBatch : gemm_batch(1, true), 0, true, VAR != 1 && VAR != 3, 0, false, false, 0, false, true,
              VAR == 3>(a, (int)blockIdx.x, smem);
}

// Two to four rows (the bulk of the large model's review passes) on a single-chunk input: the same body without the
// staging rounds for more rows and without the multi-chunk loop.  Run through the general kernel a pass of these row
// counts costs about 0.7 us more per projection (measured: one row through gemm_kernel 1018 us per T5-large pass,
// through gemm_row_kernel 911 us), which is code size and register pressure, not work.
template <int DT, int RW, int EPI, int ROPE, bool SHORT, int PS = 0>
__global__ __launch_bounds__(512) void gemm_few_kernel(BILD_GEMM_HOT_PARAMS, const GemmArgs a0) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const GemmArgs a = gemm_hot<HOT_X, DT>(a0, BILD_GEMM_HOT_NAMES);
    gemm_body<DT, RW, EPI, ROPE, 1, gemm_batch(RW, false, 1), 0, false, !SHORT, 4, false, false, PS>(a, (int)blockIdx.x, smem);
}

// A projection cut into slices of its inputs (few output features, many inputs: the FFN output projection of the
// narrow models, 64 feature tiles x 4096 inputs): blockIdx.y picks the slice, every slice writes a partial result of its own
// and the next projection adds them to the residual stream while staging.  One row (VAR as in gemm_row_kernel) or
// two to four rows (FEW, SHORT as in gemm_few_kernel).
__device__ __forceinline__ GemmArgs part_slice(const GemmArgs& a, int kt) {
    GemmArgs b = a;
    const int tps = a.W.tk / kPartSlices, ks = (int)blockIdx.y;  // (the launcher insists on ksplit == kPartSlices)
    b.k_off_tiles = ks * tps;
    b.k_len = tps * kt;
    b.x = a.x + (size_t)ks * tps * kt;
    b.out = a.out + (size_t)ks * a.part_stride;
    return b;
}
template <int DT, int VAR>
__global__ __launch_bounds__(512) void gemm_part_row_kernel(BILD_GEMM_HOT_PARAMS, const GemmArgs a0) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const GemmArgs b = part_slice(gemm_hot<HOT_X, DT>(a0, BILD_GEMM_HOT_NAMES), DT ? 32 : 16);
    gemm_body<DT, 1, EPI_PART, 0, 1, VAR ? kShortBatch : gemm_batch(1, true), 0, true, VAR != 1 && VAR != 3, 0, false, false, 0, true, false,
              VAR == 3>(b, (int)blockIdx.x, smem);
}
template <int DT, bool SHORT>
__global__ __launch_bounds__(512) void gemm_part_few_kernel(BILD_GEMM_HOT_PARAMS, const GemmArgs a0) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const GemmArgs b = part_slice(gemm_hot<HOT_X, DT>(a0, BILD_GEMM_HOT_NAMES), DT ? 32 : 16);
    gemm_body<DT, 1, EPI_PART, 0, 1, gemm_batch(1, false, 1), 0, false, !SHORT, 4, false, false, 0, true>(b, (int)blockIdx.x, smem);
}

// Output projection whose input is still in key-split attention partials (merged while staging).
template <int DT, int SPLITS, bool SHORT = false>
__global__ __launch_bounds__(512) void gemm_merge_kernel(BILD_GEMM_HOT_PARAMS, const GemmArgs a0) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const GemmArgs a = gemm_hot<HOT_MG, DT>(a0, BILD_GEMM_HOT_NAMES);
    gemm_body<DT, 1, EPI_RESID, 0, 1, gemm_batch(1, false), SPLITS, false, !SHORT>(a, (int)blockIdx.x, smem);
}

// Between kMaxRows and kDenseMinRows rows (an encoder over a source of a few hundred tokens): blockIdx.y picks a block
// of kMaxRows rows and the same body runs on it.  The blocks of one feature group re-read its weight tiles, which by
// then sit in L2 or the memory-side cache, so HBM still streams every weight about once.  At these sizes a projection
// is a GFLOP or two: too little to fill the dense-tile kernel's 64-row tiles on 256 compute units (measured on 512 rows
// of 1024..4096-wide projections: 12..40 us per launch there, 12..25 us here); longer passes go to gemm_dense.hip.
template <int DT, int RW, int EPI, int ROPE>
__global__ __launch_bounds__(512) void gemm_rows_kernel(BILD_GEMM_HOT_PARAMS, const GemmArgs a0) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const GemmArgs a = gemm_hot<HOT_X, DT>(a0, BILD_GEMM_HOT_NAMES);
    GemmArgs b = a;
    const int r0 = (int)blockIdx.y * kMaxRows;
    b.T = min(kMaxRows, a.T - r0);
    b.x = a.x + (size_t)r0 * a.ldx;
    if (a.out) b.out = a.out + (size_t)r0 * a.ldo;
    if (a.q_out) b.q_out = a.q_out + (size_t)r0 * a.i_dim;
    b.pos_add = a.pos_add + r0;
    gemm_body<DT, RW, EPI, ROPE, 2>(b, (int)blockIdx.x, smem);
}

// LDS a GEMM workgroup may ask for (a gfx950 compute unit has 160 KiB) and the share of it the staged chunk may take:
// a longer chunk means fewer chunk boundaries, at each of which the weight stream of the workgroup pauses for the staging.
constexpr int kGemmLdsLimit = 160 * 1024;
constexpr int kGemmStageBudget = 144 * 1024;
// Inputs (and input tiles) one workgroup covers: all of them, or one slice of a split projection.
static inline int eff_k(const GemmArgs& a) { return a.ksplit > 1 ? a.W.k / a.ksplit : a.W.k; }
static inline int eff_tk(const GemmArgs& a) { return a.ksplit > 1 ? a.W.tk / a.ksplit : a.W.tk; }

// Rows-per-wave, chunk length and tiles per chunk of a GEMM: what both launch-shape rules start from.
static int gemm_pick_chunks(GemmArgs& a, int dtype) {
    const int kt = dtype ? 32 : 16;
    const bool gated = a.epi == EPI_ACT && a.act != BILD_ACT_RELU;
    // A very wide LM head (250k ids) at up to 16 rows: four feature tiles per wave, so that a workgroup streams long
    // enough for the staging of its activations (the registers allow one workgroup per compute unit) to be a small share.
    // (measured: 75 -> 52 us on a 250112 x 512 head; no gain on 32128 x 1024 or 32000 x 4096)
    a.rw = gated ? 2 : (a.epi == EPI_LMHEAD && a.T <= 16 && a.W.tn >= 8192 ? 4 : 1);
    // input chunks staged in LDS: at most 96 KiB and never more than the limit leaves beside the largest
    // reduction area (8 waves), balanced so that every chunk has the same tile count +-1
    const int Tb = std::min(a.T, kMaxRows);  // rows one workgroup handles (more rows: more row blocks)
    const int budget = std::min(kGemmStageBudget, kGemmLdsLimit - gemm_tail_bytes(8, a.rw * ((Tb + 15) / 16)));
    int kc_max = budget / (4 * Tb) - 8;      // 4 bytes of LDS per staged input for either storage type
    kc_max = std::max(128, (kc_max / 128) * 128);
    const int nch = (eff_k(a) + kc_max - 1) / kc_max;
    const int kc = ((eff_k(a) + nch - 1) / nch + kt - 1) / kt * kt;
    a.kc = kc;
    const int tiles_last = (eff_k(a) - (nch - 1) * kc) / kt;
    return std::min(kc / kt, tiles_last);
}

void gemm_pick_shape(GemmArgs& a, int dtype) {
    if (a.T >= kDenseMinRows) {  // many rows (long sources, prompt prefill): the dense-tile kernel has one fixed shape
        a.wk = 1;
        a.nwv = kDenseWaves;
        a.rw = kDenseRW;
        a.kc = dense_kc(dtype);
        return;
    }
    const int tiles_chunk = gemm_pick_chunks(a, dtype);
    const int Tb = std::min(a.T, kMaxRows);
    const int nacc = a.rw * ((Tb + 15) / 16);
    // input slices per workgroup.  Latency rule (small matrices): at most one batch of tiles per wave.
    // Parallelism rule (large ones): no more slices than it takes to field about 1536 waves, so that a
    // wave streams a long contiguous run (measured best on 32128x1024, 22016x4096 and 4096x11008).
    const int batch = gemm_batch(a.rw, a.T == 1, (Tb + 15) / 16);
    int wk_lat = 1, wk_par = 1;
    while (wk_lat < 8 && eff_tk(a) / wk_lat > batch) wk_lat *= 2;
    while (wk_par < 8 && (long)a.W.tn * wk_par < 1536) wk_par *= 2;
    int wk = std::min(wk_lat, wk_par);
    while (wk > 1 && (wk * nacc > 32 || wk > tiles_chunk)) wk /= 2;
    const int row_blocks = (a.T + kMaxRows - 1) / kMaxRows;
    if (row_blocks > 1) {
        // Several row blocks: the staged activations are the larger stream, and every feature tile of a workgroup
        // reuses them, so take as many feature tiles per workgroup (8 waves) as still leave one workgroup
        // per CU; the remaining waves split the inputs.
        int wr = 8;
        while (wr > 1 && ((a.W.tn + wr * a.rw - 1) / (wr * a.rw)) * row_blocks < 256) wr /= 2;
        a.wk = 8 / wr;
        while (a.wk > 1 && a.wk > tiles_chunk) a.wk /= 2;  // (a power of two: the kernels cut the wave index by shifts)
        a.nwv = a.wk * wr;
        return;
    }
    // feature groups: as many as keep >= 512 workgroups; at least 4 waves per workgroup, 8 once a thread of a 4-wave
    // workgroup would stage more than eight pieces (staging the activations is then the longer part, and it is shared
    // by all waves; measured on 24 layers of 1024-wide projections: 4 waves win up to 8 rows, 1365 against 1490 us per
    // pass, 8 waves from 9 rows, 1505 against 1578)
    int wr = std::max(1, ((long)a.T * eff_k(a) > 8192 && a.epi != EPI_LMHEAD ? 8 : 4) / wk);
    // One row of a small matrix: fewer feature groups per workgroup while that leaves fewer than 256 workgroups - the
    // stage is bound by latency, and more compute units pulling shorten it (measured on T5-small, 96 feature tiles x 512
    // inputs: 48 workgroups of 4 waves against 96 of 2, 174.7 -> 168.2 us per step; no change at two to four rows).
    if (a.T == 1 && a.epi != EPI_LMHEAD)
        while (wr > 1 && (a.W.tn + wr * a.rw - 1) / (wr * a.rw) < 256) wr /= 2;
    for (int c = wr * 2; c * wk <= 8 && c * wk * nacc <= 32; c *= 2)
        if ((a.W.tn + c * a.rw - 1) / (c * a.rw) >= 512) wr = c;
    // Between one and two workgroups per compute unit the chip ends up half with two and half with one of them:
    // halve the workgroups instead (12288 x 4096 at one row: 384 workgroups 23.4 us, 768 of half the size 21.5 us; with
    // several rows the doubled staging costs more than the balance gains).
    const int blocks = (a.W.tn + wr * a.rw - 1) / (wr * a.rw);
    if (wr > 1 && blocks > 256 && blocks < 512 && a.epi != EPI_LMHEAD && a.T == 1) wr /= 2;
    a.wk = wk;
    a.nwv = wk * wr;
}

size_t gemm_lds_bytes(const GemmArgs& a, int dtype) {
    if (a.T >= kDenseMinRows) return dense_lds_bytes(dtype);
    const int Tb = std::min(a.T, kMaxRows);
    const int nacc = a.rw * ((Tb + 15) / 16);
    return (size_t)xs_bytes(dtype, a.kc, Tb) + gemm_tail_bytes(a.nwv, nacc);
}

size_t gemm_num_blocks(const GemmArgs& a) {
    const int per = (a.nwv / a.wk) * a.rw;
    return (size_t)(a.W.tn + per - 1) / per;
}

// The big kernels may ask for more than the default 64 KiB of dynamic LDS.
static hipError_t raise_lds_limits() {
    static hipError_t done = [] {
        const int lim = kGemmLdsLimit;
#define BILD_G1(DTV, NTV) \
    (const void*)gemm_kernel<DTV, 1, EPI_STORE, 0, NTV>, (const void*)gemm_kernel<DTV, 1, EPI_RESID, 0, NTV>, \
    (const void*)gemm_kernel<DTV, 1, EPI_QKV, 0, NTV>, (const void*)gemm_kernel<DTV, 1, EPI_QKV, 1, NTV>, \
    (const void*)gemm_kernel<DTV, 1, EPI_ACT, 0, NTV>, (const void*)gemm_kernel<DTV, 2, EPI_ACT, 0, NTV>, \
    (const void*)gemm_kernel<DTV, 1, EPI_LMHEAD, 0, NTV>
#define BILD_G(DTV) BILD_G1(DTV, 1), BILD_G1(DTV, 2), BILD_R(DTV)
#define BILD_R(DTV) \
    (const void*)gemm_row_kernel<DTV, 1, EPI_STORE, 0>, (const void*)gemm_row_kernel<DTV, 1, EPI_RESID, 0>, \
    (const void*)gemm_row_kernel<DTV, 1, EPI_QKV, 0>, (const void*)gemm_row_kernel<DTV, 1, EPI_QKV, 1>, \
    (const void*)gemm_row_kernel<DTV, 1, EPI_ACT, 0>, (const void*)gemm_row_kernel<DTV, 2, EPI_ACT, 0>, \
    (const void*)gemm_row_kernel<DTV, 1, EPI_LMHEAD, 0>, (const void*)gemm_row_kernel<DTV, 4, EPI_LMHEAD, 0>, \
    (const void*)gemm_row_kernel<DTV, 1, EPI_LMHEAD, 0, 2>, \
    (const void*)gemm_row_kernel<DTV, 1, EPI_STORE, 0, 1>, (const void*)gemm_row_kernel<DTV, 1, EPI_RESID, 0, 1>, \
    (const void*)gemm_row_kernel<DTV, 1, EPI_QKV, 0, 1>, (const void*)gemm_row_kernel<DTV, 1, EPI_QKV, 1, 1>, \
    (const void*)gemm_row_kernel<DTV, 1, EPI_ACT, 0, 1>, \
    (const void*)gemm_row_kernel<DTV, 1, EPI_STORE, 0, 3>, (const void*)gemm_row_kernel<DTV, 1, EPI_RESID, 0, 3>, \
    (const void*)gemm_row_kernel<DTV, 1, EPI_QKV, 0, 3>, (const void*)gemm_row_kernel<DTV, 1, EPI_QKV, 1, 3>, \
    (const void*)gemm_row_kernel<DTV, 1, EPI_ACT, 0, 3>, \
    (const void*)gemm_row_kernel<DTV, 1, EPI_STORE, 0, 2>, (const void*)gemm_row_kernel<DTV, 1, EPI_RESID, 0, 2>, \
    (const void*)gemm_row_kernel<DTV, 1, EPI_QKV, 0, 2>, (const void*)gemm_row_kernel<DTV, 1, EPI_QKV, 1, 2>, \
    (const void*)gemm_row_kernel<DTV, 1, EPI_ACT, 0, 2>, \
    (const void*)gemm_row_kernel<DTV, 2, EPI_ACT, 0, 1>, (const void*)gemm_row_kernel<DTV, 2, EPI_ACT, 0, 2>, \
    (const void*)gemm_row_embed_kernel<DTV, 0, 0>, (const void*)gemm_row_embed_kernel<DTV, 0, 1>, (const void*)gemm_row_embed_kernel<DTV, 0, 2>, \
    (const void*)gemm_row_embed_kernel<DTV, 1, 0>, (const void*)gemm_row_embed_kernel<DTV, 1, 1>, (const void*)gemm_row_embed_kernel<DTV, 1, 2>, \
    (const void*)gemm_few_kernel<DTV, 1, EPI_STORE, 0, true>, (const void*)gemm_few_kernel<DTV, 1, EPI_RESID, 0, true>, \
    (const void*)gemm_few_kernel<DTV, 1, EPI_QKV, 0, true>, (const void*)gemm_few_kernel<DTV, 1, EPI_QKV, 1, true>, \
    (const void*)gemm_few_kernel<DTV, 1, EPI_ACT, 0, true>, \
    (const void*)gemm_few_kernel<DTV, 1, EPI_STORE, 0, false>, (const void*)gemm_few_kernel<DTV, 1, EPI_RESID, 0, false>, \
    (const void*)gemm_few_kernel<DTV, 1, EPI_QKV, 0, false>, (const void*)gemm_few_kernel<DTV, 1, EPI_QKV, 1, false>, \
    (const void*)gemm_few_kernel<DTV, 1, EPI_ACT, 0, false>, \
    (const void*)gemm_kernel<DTV, 1, EPI_STORE, 0, 1, true>, (const void*)gemm_kernel<DTV, 1, EPI_RESID, 0, 1, true>, \
    (const void*)gemm_kernel<DTV, 1, EPI_QKV, 0, 1, true>, (const void*)gemm_kernel<DTV, 1, EPI_QKV, 1, 1, true>, \
    (const void*)gemm_kernel<DTV, 1, EPI_ACT, 0, 1, true>, \
    (const void*)gemm_kernel<DTV, 4, EPI_LMHEAD, 0, 1>, \
    (const void*)gemm_rows_kernel<DTV, 1, EPI_STORE, 0>, (const void*)gemm_rows_kernel<DTV, 1, EPI_RESID, 0>, \
    (const void*)gemm_rows_kernel<DTV, 1, EPI_QKV, 0>, (const void*)gemm_rows_kernel<DTV, 1, EPI_QKV, 1>, \
    (const void*)gemm_rows_kernel<DTV, 1, EPI_ACT, 0>, (const void*)gemm_rows_kernel<DTV, 2, EPI_ACT, 0>
        const void* fns[] = {BILD_G(0), BILD_G(1),
                             (const void*)gemm_merge_kernel<0, 2>, (const void*)gemm_merge_kernel<0, 4>,
                             (const void*)gemm_merge_kernel<0, 8>, (const void*)gemm_merge_kernel<1, 2>,
                             (const void*)gemm_merge_kernel<1, 4>, (const void*)gemm_merge_kernel<1, 8>,
                             (const void*)gemm_merge_kernel<0, 2, true>, (const void*)gemm_merge_kernel<0, 4, true>,
                             (const void*)gemm_merge_kernel<0, 8, true>, (const void*)gemm_merge_kernel<1, 2, true>,
                             (const void*)gemm_merge_kernel<1, 4, true>, (const void*)gemm_merge_kernel<1, 8, true>,
                             };
#undef BILD_G1
#undef BILD_G
#undef BILD_R
        for (const void* f : fns) {
            hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, lim);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }();
    return done;
}

hipError_t kernels_init() {
    if (hipError_t e = raise_lds_limits(); e != hipSuccess) return e;
    if (hipError_t e = gemm_pre_init(); e != hipSuccess) return e;
    return attention_init();
}

// Split projections (EPI_PART) and their readers (pn > 0): one to four rows, one chunk of inputs.
static hipError_t launch_gemm_split(const GemmArgs& a, int dtype, hipStream_t st) {
    const size_t smem = gemm_lds_bytes(a, dtype);
    const int kk = eff_k(a), tk = eff_tk(a);
    const bool one_chunk = kk <= a.kc;
    const int per_wave = (tk + a.wk - 1) / a.wk;
    const bool exact8 = a.rw == 1 && tk == kShortBatch * a.wk;  // every wave has exactly one batch of tiles
    const int n4 = kk / 4, nthr = 64 * a.nwv;
    if (a.T < 1 || a.T > 4 || !one_chunk || (a.rw != 1 && !(a.rw == 2 && a.epi == EPI_ACT)) || a.mg_splits > 1 || a.xb_hi || a.nx_hi)
        return hipErrorInvalidValue;
    // the staging paths these kernels keep: one row with at most two pieces per thread; two to four rows with whole
    // wavefront-wide rows and at most four pieces per thread
    if (a.T == 1 ? n4 > 2 * nthr : ((n4 & 63) != 0 || a.T * n4 > 4 * nthr)) return hipErrorInvalidValue;
    const dim3 block(nthr);
    if (a.epi == EPI_PART) {
        if (a.ksplit != kPartSlices || a.W.tk % a.ksplit || a.pn > 0 || !a.out) return hipErrorInvalidValue;
        const dim3 grid((unsigned)gemm_num_blocks(a), (unsigned)a.ksplit);
#define BILD_PK(DTV)                                                                                              \
    do {                                                                                                          \
        if (a.T == 1 && exact8) hipLaunchKernelGGL((gemm_part_row_kernel<DTV, 3>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
        else if (a.T == 1 && per_wave <= kShortBatch) hipLaunchKernelGGL((gemm_part_row_kernel<DTV, 1>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
        else if (a.T == 1 && per_wave <= 2 * kShortBatch) hipLaunchKernelGGL((gemm_part_row_kernel<DTV, 2>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
        else if (a.T == 1) hipLaunchKernelGGL((gemm_part_row_kernel<DTV, 0>), grid, block, smem, st, BILD_GEMM_HOT(a), a);          \
        else if (per_wave <= gemm_batch(1, false)) hipLaunchKernelGGL((gemm_part_few_kernel<DTV, true>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
        else hipLaunchKernelGGL((gemm_part_few_kernel<DTV, false>), grid, block, smem, st, BILD_GEMM_HOT(a), a);                    \
    } while (0)
        if (dtype) BILD_PK(1); else BILD_PK(0);
#undef BILD_PK
        return hipGetLastError();
    }
    if (a.pn < 1 || !a.px || !a.x_out || a.x_out == a.x || a.ksplit > 1) return hipErrorInvalidValue;
    // the kernels derive the stride of the partial results from ldx and get x_out as a 32-bit offset from x (gemm_hot)
    if (a.px_stride != (int64_t)kMaxRows * a.ldx || (int64_t)(a.x_out - a.x) != (int64_t)(int)(a.x_out - a.x)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)gemm_num_blocks(a));
    if (a.epi == EPI_STORE || a.epi == EPI_ACT) {
        // readers of one partial result per head (attention fused with its output projection): single-row passes
        if (a.T != 1 || a.pn != kMaxHeadParts) return hipErrorInvalidValue;
        constexpr int PH = kMaxHeadParts;
#define BILD_RH(DTV)                                                                                              \
    do {                                                                                                          \
        if (a.epi == EPI_ACT && a.rw == 2) {                                                                      \
            if (per_wave <= kShortBatch / 2) hipLaunchKernelGGL((gemm_row_kernel<DTV, 2, EPI_ACT, 0, 1, PH>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
            else if (per_wave <= kShortBatch || (per_wave % 4 == 0 && per_wave % 6 != 0))                         \
                hipLaunchKernelGGL((gemm_row_kernel<DTV, 2, EPI_ACT, 0, 2, PH>), grid, block, smem, st, BILD_GEMM_HOT(a), a);       \
            else hipLaunchKernelGGL((gemm_row_kernel<DTV, 2, EPI_ACT, 0, 0, PH>), grid, block, smem, st, BILD_GEMM_HOT(a), a);      \
        } else if (a.epi == EPI_ACT) {                                                                            \
            if (exact8) hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPI_ACT, 0, 3, PH>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
            else if (per_wave <= kShortBatch) hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPI_ACT, 0, 1, PH>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
            else if (per_wave <= 2 * kShortBatch || (per_wave % kShortBatch == 0 && per_wave % 12 != 0))          \
                hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPI_ACT, 0, 2, PH>), grid, block, smem, st, BILD_GEMM_HOT(a), a);       \
            else hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPI_ACT, 0, 0, PH>), grid, block, smem, st, BILD_GEMM_HOT(a), a);      \
        } else {                                                                                                  \
            if (exact8) hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPI_STORE, 0, 3, PH>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
            else if (per_wave <= kShortBatch) hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPI_STORE, 0, 1, PH>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
            else if (per_wave <= 2 * kShortBatch || (per_wave % kShortBatch == 0 && per_wave % 12 != 0))          \
                hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPI_STORE, 0, 2, PH>), grid, block, smem, st, BILD_GEMM_HOT(a), a);     \
            else hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPI_STORE, 0, 0, PH>), grid, block, smem, st, BILD_GEMM_HOT(a), a);    \
        }                                                                                                         \
    } while (0)
        if (dtype) BILD_RH(1); else BILD_RH(0);
#undef BILD_RH
        return hipGetLastError();
    }
    if (a.pn != kPartSlices) return hipErrorInvalidValue;
    constexpr int PSV = kPartSlices;
#define BILD_RD1(DTV, EPIV, ROPEV) /* one row */                                                                 \
    do {                                                                                                          \
        if (exact8)                                                                                               \
            hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPIV, ROPEV, 3, PSV>), grid, block, smem, st, BILD_GEMM_HOT(a), a);         \
        else if (per_wave <= kShortBatch)                                                                         \
            hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPIV, ROPEV, 1, PSV>), grid, block, smem, st, BILD_GEMM_HOT(a), a);         \
        else if (per_wave <= 2 * kShortBatch || (per_wave % kShortBatch == 0 && per_wave % 12 != 0))              \
            hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPIV, ROPEV, 2, PSV>), grid, block, smem, st, BILD_GEMM_HOT(a), a);         \
        else                                                                                                      \
            hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPIV, ROPEV, 0, PSV>), grid, block, smem, st, BILD_GEMM_HOT(a), a);         \
    } while (0)
#define BILD_RDF(DTV, ROPEV) /* two to four rows: the first projection of a layer only */                         \
    do {                                                                                                          \
        if (per_wave <= gemm_batch(1, false))                                                                     \
            hipLaunchKernelGGL((gemm_few_kernel<DTV, 1, EPI_QKV, ROPEV, true, PSV>), grid, block, smem, st, BILD_GEMM_HOT(a), a);   \
        else                                                                                                      \
            hipLaunchKernelGGL((gemm_few_kernel<DTV, 1, EPI_QKV, ROPEV, false, PSV>), grid, block, smem, st, BILD_GEMM_HOT(a), a);  \
    } while (0)
#define BILD_RDD(DTV)                                                                                             \
    if (a.epi == EPI_QKV && a.T == 1) { if (a.rope) BILD_RD1(DTV, EPI_QKV, 1); else BILD_RD1(DTV, EPI_QKV, 0); }  \
    else if (a.epi == EPI_QKV) { if (a.rope) BILD_RDF(DTV, 1); else BILD_RDF(DTV, 0); }                           \
    else if (a.epi == EPI_LMHEAD && a.T == 1) BILD_RD1(DTV, EPI_LMHEAD, 0);                                       \
    else return hipErrorInvalidValue;
    if (dtype) { BILD_RDD(1) } else { BILD_RDD(0) }
#undef BILD_RDD
#undef BILD_RDF
#undef BILD_RD1
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs& a, int dtype, hipStream_t st) {
    if (hipError_t e = raise_lds_limits(); e != hipSuccess) return e;
    if (a.T >= kDenseMinRows) return launch_gemm_dense(a, dtype, st);
    if (a.wk < 1 || a.wk > 8 || (a.wk & (a.wk - 1)) || a.nwv % a.wk || a.nwv > 8) return hipErrorInvalidValue;  // (gemm_hot_geom)
    if (a.xb_hi || a.nx_hi) return dtype ? launch_gemm_pre(a, st) : hipErrorInvalidValue;
    const size_t smem = gemm_lds_bytes(a, dtype);
    const unsigned row_blocks = (unsigned)((a.T + kMaxRows - 1) / kMaxRows);
    if (row_blocks > 1 && a.epi == EPI_LMHEAD) return hipErrorInvalidValue;  // softmax partials are per pass
    if ((a.gain != nullptr) != (a.epi != EPI_RESID && a.epi != EPI_PART)) return hipErrorInvalidValue;  // the kernels fix the norm by the epilogue
    if (a.e_w) {
        // input row gathered from the embedding matrix: one row, one chunk, the plain first projection of a layer
        const int per_wave = (a.W.tk + a.wk - 1) / a.wk;
        if (a.T != 1 || a.epi != EPI_QKV || a.rw != 1 || a.W.k > a.kc || a.pn > 0 || a.mg_splits > 1 || !a.x_out || a.x != a.x_out ||
            !a.e_tokens || !a.e_base_ptr || a.e_vocab < 1 || a.e_shift < 0 || a.e_shift >= a.e_vocab || a.e_tk * (dtype ? 32 : 16) != a.W.k)
            return hipErrorInvalidValue;
        const dim3 grid((unsigned)gemm_num_blocks(a)), block(64 * a.nwv);
#define BILD_EM(DTV, ROPEV)                                                                                                       \
    do {                                                                                                                            \
        if (a.W.tk == kShortBatch * a.wk) hipLaunchKernelGGL((gemm_row_embed_kernel<DTV, ROPEV, 3>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
        else if (per_wave <= kShortBatch) hipLaunchKernelGGL((gemm_row_embed_kernel<DTV, ROPEV, 1>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
        else if (per_wave <= 2 * kShortBatch || (per_wave % kShortBatch == 0 && per_wave % 12 != 0))                                \
            hipLaunchKernelGGL((gemm_row_embed_kernel<DTV, ROPEV, 2>), grid, block, smem, st, BILD_GEMM_HOT(a), a);                 \
        else hipLaunchKernelGGL((gemm_row_embed_kernel<DTV, ROPEV, 0>), grid, block, smem, st, BILD_GEMM_HOT(a), a);                \
    } while (0)
        if (dtype) { if (a.rope) BILD_EM(1, 1); else BILD_EM(1, 0); }
        else { if (a.rope) BILD_EM(0, 1); else BILD_EM(0, 0); }
#undef BILD_EM
        return hipGetLastError();
    }
    if (a.epi == EPI_PART || a.pn > 0) return launch_gemm_split(a, dtype, st);
    if (a.mg_splits > 1) {
        // merged staging: 2, 4 or 8 splits, up to 16 rows, one (row, head) pair per thread, weights in the reduction area
        const int sp = a.mg_splits, npairs = a.T * a.mg_heads;
        if ((sp != 2 && sp != 4 && sp != 8) || a.gain || a.T > 16 || a.epi != EPI_RESID || a.rw != 1 || a.mg_heads < 1 ||
            npairs > 64 * a.nwv || (size_t)npairs * sp * 4 > (size_t)gemm_red_bytes(a.nwv, 1))
            return hipErrorInvalidValue;
        const dim3 grid1((unsigned)gemm_num_blocks(a)), block1(64 * a.nwv);
#define BILD_MG(DTV, SH)                                                                       \
    do {                                                                                        \
        if (sp == 2) hipLaunchKernelGGL((gemm_merge_kernel<DTV, 2, SH>), grid1, block1, smem, st, BILD_GEMM_HOT_MG(a), a); \
        else if (sp == 4) hipLaunchKernelGGL((gemm_merge_kernel<DTV, 4, SH>), grid1, block1, smem, st, BILD_GEMM_HOT_MG(a), a); \
        else hipLaunchKernelGGL((gemm_merge_kernel<DTV, 8, SH>), grid1, block1, smem, st, BILD_GEMM_HOT_MG(a), a);   \
    } while (0)
        // (one batch of tiles per wave at most: no second weight buffer, see gemm_row_kernel)
        const bool sh = a.W.k <= a.kc && (a.W.tk + a.wk - 1) / a.wk <= gemm_batch(1, false);
        if (dtype) { if (sh) BILD_MG(1, true); else BILD_MG(1, false); }
        else { if (sh) BILD_MG(0, true); else BILD_MG(0, false); }
#undef BILD_MG
        return hipGetLastError();
    }
    const dim3 grid((unsigned)gemm_num_blocks(a), row_blocks), block(64 * a.nwv);
    // tiles the busiest wave has: picks the batch geometry (see gemm_row_kernel)
    const bool one_chunk = a.W.k <= a.kc;
    const int per_wave = (a.W.tk + a.wk - 1) / a.wk;
    // two to four rows, one chunk, and either ragged rows (dealt row by row) or at most four staged pieces per thread
    const int n4 = a.W.k / 4;
    const bool few_ok = a.T >= 2 && a.T <= 4 && one_chunk && ((n4 & 63) != 0 || a.T * n4 <= 4 * 64 * a.nwv);
#define BILD_L(DTV, RWV, EPIV, ROPEV)                                                              \
    do {                                                                                            \
        if (row_blocks > 1)                                                                         \
            hipLaunchKernelGGL((gemm_rows_kernel<DTV, RWV, EPIV, ROPEV>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
        else if (a.T == 1 && RWV == 2 && one_chunk && per_wave <= kShortBatch / 2)                  \
            hipLaunchKernelGGL((gemm_row_kernel<DTV, 2, EPI_ACT, 0, 1>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
        else if (a.T == 1 && RWV == 2 && one_chunk && (per_wave <= kShortBatch || (per_wave % 4 == 0 && per_wave % 6 != 0))) \
            hipLaunchKernelGGL((gemm_row_kernel<DTV, 2, EPI_ACT, 0, 2>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
        else if (a.T == 1 && RWV == 1 && one_chunk && a.W.tk == kShortBatch * a.wk)                 \
            hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPIV, ROPEV, 3>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
        else if (a.T == 1 && RWV == 1 && one_chunk && per_wave <= kShortBatch)                      \
            hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPIV, ROPEV, 1>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
        else if (a.T == 1 && RWV == 1 && one_chunk && (per_wave <= 2 * kShortBatch || (per_wave % kShortBatch == 0 && per_wave % 12 != 0))) \
            hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPIV, ROPEV, 2>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
        else if (a.T == 1 && one_chunk)                                                             \
            hipLaunchKernelGGL((gemm_row_kernel<DTV, RWV, EPIV, ROPEV>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
        else if (a.T > 16)                                                                          \
            hipLaunchKernelGGL((gemm_kernel<DTV, RWV, EPIV, ROPEV, 2>), grid, block, smem, st, BILD_GEMM_HOT(a), a);  \
        else if (RWV == 1 && few_ok && per_wave <= gemm_batch(1, false))                            \
            hipLaunchKernelGGL((gemm_few_kernel<DTV, 1, EPIV, ROPEV, true>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
        else if (RWV == 1 && few_ok)                                                                \
            hipLaunchKernelGGL((gemm_few_kernel<DTV, 1, EPIV, ROPEV, false>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
        else if (RWV == 1 && one_chunk && per_wave <= gemm_batch(1, false))                         \
            hipLaunchKernelGGL((gemm_kernel<DTV, 1, EPIV, ROPEV, 1, true>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
        else                                                                                        \
            hipLaunchKernelGGL((gemm_kernel<DTV, RWV, EPIV, ROPEV, 1>), grid, block, smem, st, BILD_GEMM_HOT(a), a);  \
    } while (0)
#define BILD_D(DTV)                                                              \
    switch (a.epi) {                                                             \
        case EPI_STORE: BILD_L(DTV, 1, EPI_STORE, 0); break;                     \
        case EPI_RESID: BILD_L(DTV, 1, EPI_RESID, 0); break;                     \
        case EPI_QKV:                                                            \
            if (a.rope) BILD_L(DTV, 1, EPI_QKV, 1); else BILD_L(DTV, 1, EPI_QKV, 0); \
            break;                                                               \
        case EPI_ACT:                                                            \
            if (a.rw == 2) BILD_L(DTV, 2, EPI_ACT, 0); else BILD_L(DTV, 1, EPI_ACT, 0); \
            break;                                                               \
        case EPI_LMHEAD:                                                         \
            if (a.rw == 4 && a.T == 1 && one_chunk)                              \
                hipLaunchKernelGGL((gemm_row_kernel<DTV, 4, EPI_LMHEAD, 0>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
            else if (a.rw == 4 && a.T <= 16)                                     \
                hipLaunchKernelGGL((gemm_kernel<DTV, 4, EPI_LMHEAD, 0, 1>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
            else if (a.rw != 1)                                                  \
                return hipErrorInvalidValue;                                     \
            else if (a.T == 1 && one_chunk && per_wave <= 32 && per_wave % kShortBatch == 0) /* batches of 8 fit exactly */ \
                hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPI_LMHEAD, 0, 2>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
            else if (a.T == 1 && one_chunk)                                      \
                hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPI_LMHEAD, 0>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
            else if (a.T > 16)                                                   \
                hipLaunchKernelGGL((gemm_kernel<DTV, 1, EPI_LMHEAD, 0, 2>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
            else                                                                 \
                hipLaunchKernelGGL((gemm_kernel<DTV, 1, EPI_LMHEAD, 0, 1>), grid, block, smem, st, BILD_GEMM_HOT(a), a); \
            break;                                                               \
        default: return hipErrorInvalidValue;                                    \
    }
    if (dtype) { BILD_D(1) } else { BILD_D(0) }
#undef BILD_D
#undef BILD_L
    return hipGetLastError();
}


// =====================================================================================
// Embedding gather from the tiled matrix (+ sinusoidal position).
// =====================================================================================
template <int DT>
__device__ __forceinline__ void embed_body(const EmbedArgs& a, const int t) {
    constexpr int KT = DT ? 32 : 16, PL = KT / 4;
    const int base = (a.base_ptr ? *a.base_ptr : 0) + a.base_add;
    const int tok = a.tokens[base + t];
    const int row = (int)(((long long)tok + a.tie_shift) % a.vocab);
    const int pos = base + t;
    const double lg = log2(10000.0);
    float ss = 0.f;
    for (int k = threadIdx.x; k < a.d; k += blockDim.x) {
        const size_t tile = (size_t)(row >> 4) * a.E.tk + (k / KT);
        const int ln = (row & 15) + 16 * ((k % KT) / PL), j = k % PL;
        const char* p = (const char*)a.E.w + tile * kTileBytes + ln * 16;
        float v = DT ? bf2f(((const uint16_t*)p)[j]) : ((const float*)p)[j];
        // one fused multiply-add (value times scale plus the position term), spelled out so that the projection that
        // gathers its own input row (gemm_body, EMB) rounds the same way
        float pterm = 0.f;
        if (a.sinusoidal) {
            if (a.pe) {
                pterm = a.pe[(size_t)pos * a.d + k];
            } else {
                const double ang = (double)pos * exp2(-(double)(2 * (k >> 1)) / (double)a.d * lg);
                pterm = (float)((k & 1) ? cos(ang) : sin(ang));
            }
        }
        v = __builtin_fmaf(v, a.embed_scale, pterm);
        st_act(a.x + (size_t)t * a.d + k, v);
        if (a.nx_hi) {
            uint32_t hi, lo;
            split_bf16x2(v * a.nx_gain[k], 0.f, hi, lo);
            st_u16(a.nx_hi + (size_t)t * a.d + k, (uint16_t)hi);
            st_u16(a.nx_lo + (size_t)t * a.d + k, (uint16_t)lo);
            ss += v * v;
        }
    }
    if (a.nx_hi) {  // (uniform) one part per wave
        const float tot = wave_sum(ss);
        if ((threadIdx.x & 63) == 0) st_act(a.nx_ssq + (size_t)(threadIdx.x >> 6) * kMaxRows + t, tot);
    }
}

template <int DT>
__global__ __launch_bounds__(256) void embed_kernel(const EmbedArgs a) { embed_body<DT>(a, (int)blockIdx.x); }

__global__ __launch_bounds__(256) void pe_table_kernel(float* table, int d) {
    const int pos = (int)blockIdx.x;
    const double lg = log2(10000.0);
    for (int k = threadIdx.x; k < d; k += blockDim.x) {
        const double ang = (double)pos * exp2(-(double)(2 * (k >> 1)) / (double)d * lg);
        table[(size_t)pos * d + k] = (float)((k & 1) ? cos(ang) : sin(ang));
    }
}

hipError_t launch_pe_table(float* table, int positions, int d, hipStream_t st) {
    if (!table || positions < 1 || d < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(pe_table_kernel, dim3(positions), dim3(256), 0, st, table, d);
    return hipGetLastError();
}

hipError_t launch_embed(const EmbedArgs& a, int dtype, hipStream_t st) {
    if (dtype)
        hipLaunchKernelGGL(embed_kernel<1>, dim3(a.T), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(embed_kernel<0>, dim3(a.T), dim3(256), 0, st, a);
    return hipGetLastError();
}


__global__ __launch_bounds__(256) void row_copy_kernel(const RowCopyArgs a) {
    const int t = (int)blockIdx.x;
    const float4* src = (const float4*)(a.src + (size_t)((a.src_row_ptr ? *a.src_row_ptr : 0) + a.src_row_add + t) * a.d);
    float4* dst = (float4*)(a.dst + (size_t)((a.dst_row_ptr ? *a.dst_row_ptr : 0) + a.dst_row_add + t) * a.d);
    for (int i = threadIdx.x; i < a.d / 4; i += blockDim.x) dst[i] = src[i];
}

hipError_t launch_row_copy(const RowCopyArgs& a, hipStream_t st) {
    if (a.T < 1 || a.d % 4) return hipErrorInvalidValue;
    hipLaunchKernelGGL(row_copy_kernel, dim3(a.T), dim3(256), 0, st, a);
    return hipGetLastError();
}



}  // namespace bild
