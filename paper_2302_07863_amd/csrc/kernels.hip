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
//   finish_kernel    merges the LM-head partial statistics and applies the fallback /
//                    rollback policy (Sections 3.3, 3.4; Algorithm 1), committing y and
//                    the cache lengths on the device.
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

namespace bild {

// =====================================================================================
// Skinny GEMM.  A workgroup has nwv = wk * wr wavefronts arranged as wr feature groups
// x wk input slices; each wave owns RW feature tiles (16 features each) and walks the
// input tiles of its slice, U tiles per batch so that one batch of loads covers one
// round trip to HBM.  Weights do not depend on the activations: the first two batches
// are requested right behind the activation loads and before anything is waited for,
// so the conversion of the activations, the barrier and the residual read all overlap
// with the weights' trip from memory.  LDS layout (dynamic):
//   (at most 8 waves per workgroup, so that a wave may use 256 registers)
//   [0, xs)            staged activations of the current input chunk
//   red                cross-wave partial sums when wk > 1   (nwv x nacc x 64 float4)
//   ssq[nwv][32]       per-wave sums of squares for the RMSNorm
//   rs[32]             per-row 1/rms
//   wstat[nwv][32]     per-wave softmax partials (LM head)
//   zblk               64 bytes of zeros
// =====================================================================================
// weight tiles a wave loads per batch (split over its RW feature tiles); two batches are in flight
// (12 in the single-row kernel; 8 with several rows, whose staging needs the registers; 4 above 16 rows, where the
// second set of row tiles needs more and the per-wave tile counts of the row-block launches - 4, 8, 16, 32 - then
// split into whole batches; see gemm_row_kernel on what padding slots cost)
__host__ __device__ constexpr int gemm_batch(int rw, bool one_row, int nt = 1) { return (one_row ? 12 : (nt > 1 ? 4 : 8)) / rw; }

__host__ __device__ inline int xs_row_stride(int dt, int kc) { return dt ? (kc + 8) * 2 : (kc + 4) * 4; }
__host__ __device__ inline int xs_bytes(int dt, int kc, int T) { return T * xs_row_stride(dt, kc) * (dt ? 2 : 1); }
__host__ __device__ inline int gemm_red_bytes(int nwv, int nacc) { return nwv * nacc * 64 * 16; }
__host__ __device__ inline int gemm_tail_bytes(int nwv, int nacc) {
    return gemm_red_bytes(nwv, nacc) + nwv * 32 * 4 + 32 * 4 + nwv * 32 * 16 + 64;
}

// `vblock` is the index of the feature-tile group this workgroup handles (blockIdx.x); `smem` is its dynamic LDS.
template <int DT, int RW, int EPI, int ROPE, int NT, int U = gemm_batch(RW, false, NT), int MG = 0,
          bool ONE = false, bool TWO = true, int TCAP = 0>
__device__ __forceinline__ void gemm_body(const GemmArgs& a, const int vblock, char* smem) {
    constexpr int KT = DT ? 32 : 16;
    // the wave index through readfirstlane: the compiler then knows that it - and every tile index, weight address and
    // range test derived from it - is the same in all lanes, and keeps them in scalar registers
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nthr = blockDim.x, NWV = nthr >> 6;
    const int T = ONE ? 1 : a.T, K = a.W.k, KC = a.kc;
    const int WK = a.wk, WR = NWV / WK;
    const int wkid = wave % WK, wrid = wave / WK;
    const int tile0 = (vblock * WR + wrid) * RW;
    const int nacc = RW * NT;
    const int rstride = xs_row_stride(DT, KC);
    char* xs_hi = smem;
    char* xs_lo = smem + T * rstride;  // bf16 only
    char* tail = smem + xs_bytes(DT, KC, T);
    f32x4* red = (f32x4*)tail;
    float* ssq = (float*)(tail + gemm_red_bytes(NWV, nacc));
    float* rs = ssq + NWV * 32;
    StatPart* wstat = (StatPart*)(rs + 32);
    char* zblk = (char*)(wstat + NWV * 32);  // 64 bytes of zeros: the activation operand of a tile past the range

    constexpr int epi = EPI;
    constexpr bool rope = ROPE != 0;
    // Every projection that adds to the residual stream reads un-normalised input and every other one reads through an
    // RMSNorm, so the presence of the norm is a compile-time fact (the launcher rejects anything else); a run-time
    // test here would make the gain loads conditional.
    constexpr bool norm = EPI != EPI_RESID;
    const bool few = T < 4;  // few rows: all waves share each row and split it along k
    const bool owner = (wkid == 0);
    bool valid[RW];
    const char* wbase[RW];
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        valid[r] = tile0 + r < a.W.tn;
        wbase[r] = (const char*)a.W.w + ((size_t)min(tile0 + r, a.W.tn - 1) * a.W.tk) * kTileBytes;  // scalar; the lane part is added per load
    }
    const int tok_l = lane & 15, kq = lane >> 4;

    // ---- weight tiles: two register buffers of U tiles each, requested without any guard ----
    // A tile past the wave's range is read from a clamped (valid) address and cancelled on the activation
    // side (compute() reads a block of zeros for it), so no instruction touches a weight register between
    // its load and its MFMA, and the requests of a batch stay in flight across everything in between.
    // The memory counter retires loads in the order they were issued: whatever is needed first is requested
    // first.  One-chunk launches (the latency-bound ones) therefore request the activations, then both weight
    // buffers, and only then wait for the activations; the weights arrive while those are converted.
    uint4 B0[RW][U], B1[RW][U];
    const int S = U * WK;  // tiles between consecutive batches of this wave
    const unsigned lane16 = (unsigned)lane * 16u;  // scalar base + 32-bit lane offset: one address register for all loads
    auto request = [&](uint4 (&B)[RW][U], int kt_abs, int kt_end) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int ktc = min(kt_abs + u * WK, kt_end - 1);
#pragma unroll
            for (int r = 0; r < RW; ++r) B[r][u] = *(const uint4*)(wbase[r] + (size_t)ktc * kTileBytes + lane16);
        }
    };

    // residual values: unconditional loads from clamped addresses (a conditional load would have to be waited
    // for where the branches join, that is, here)
    float4 old[RW][2];
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) old[r][nt] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (epi == EPI_RESID) {
#pragma unroll
        for (int r = 0; r < RW; ++r)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                old[r][nt] = ld_act4(a.out + (size_t)min(nt * 16 + tok_l, T - 1) * a.ldo + min(tile0 + r, a.W.tn - 1) * 16 + kq * 4);
    }

    const int pos0 = (a.pos_ptr ? *a.pos_ptr : 0) + a.pos_add;
    int tgt[2] = {-1, -1};
    if (epi == EPI_LMHEAD) {
        const int ylen = *a.ylen_ptr;
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const int ti = pos0 + nt * 16 + tok_l + 1;
            if (nt * 16 + tok_l < T && ti < ylen) tgt[nt] = a.y[ti];
        }
    }

    if (lane < 32) ssq[wave * 32 + lane] = 0.f;  // each wave owns (and later accumulates into) its own row
    if (tid < 4) ((uint4*)zblk)[tid] = make_uint4(0u, 0u, 0u, 0u);

    // up to 16 rows: two accumulators per output tile (bf16: one for the high parts, one for the low parts of the
    // activations), so that consecutive MFMAs do not wait for each other; they are added once at the end.  More rows
    // have two independent tiles anyway.
    f32x4 acc[RW][2], acc2[RW][2];
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[r][j] = acc2[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int zoff = (int)(zblk - xs_hi) + kq * 16;
    auto compute = [&](const uint4 (&At)[RW], int ktl, bool ok) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            // rows past T read a valid row instead: an MFMA column only feeds its own output column,
            // and those columns are never stored
            const int t = min(nt * 16 + tok_l, T - 1);
            if (DT) {
                const int off = ok ? t * rstride + (ktl * 32 + kq * 8) * 2 : zoff;
                const int offl = ok ? off + T * rstride : zoff;
                const uint4 bh = *(const uint4*)(xs_hi + off);
                const uint4 bl = *(const uint4*)(xs_hi + offl);
                const bf16x8 Bh = __builtin_bit_cast(bf16x8, bh), Bl = __builtin_bit_cast(bf16x8, bl);
#pragma unroll
                for (int r = 0; r < RW; ++r) {
                    const bf16x8 Aw = __builtin_bit_cast(bf16x8, At[r]);
                    acc[r][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Aw, Bh, acc[r][nt], 0, 0, 0);
                    if (NT == 1) acc2[r][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Aw, Bl, acc2[r][nt], 0, 0, 0);
                    else acc[r][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Aw, Bl, acc[r][nt], 0, 0, 0);
                }
            } else {
                const int off = ok ? t * rstride + (ktl * 16 + kq * 4) * 4 : zoff;
                const float4 b = *(const float4*)(xs_hi + off);
                const float bb[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
                for (int r = 0; r < RW; ++r) {
                    const float aa[4] = {__uint_as_float(At[r].x), __uint_as_float(At[r].y),
                                         __uint_as_float(At[r].z), __uint_as_float(At[r].w)};
#pragma unroll
                    for (int j = 0; j < 4; j += 2) {
                        acc[r][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(aa[j], bb[j], acc[r][nt], 0, 0, 0);
                        if (NT == 1) acc2[r][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(aa[j + 1], bb[j + 1], acc2[r][nt], 0, 0, 0);
                        else acc[r][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(aa[j + 1], bb[j + 1], acc[r][nt], 0, 0, 0);
                    }
                }
            }
        }
    };
    // one batch against the chunk staged in LDS; kt is the wave's first tile of the batch within the chunk
    auto compute_batch = [&](uint4 (&B)[RW][U], int kt, int nkt) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint4 At[RW];
#pragma unroll
            for (int r = 0; r < RW; ++r) At[r] = B[r][u];
            compute(At, kt + u * WK, kt + u * WK < nkt);
        }
    };

    // ---- stage x[:, k0 : k0+kc_len] (times the norm gain) into LDS ----
    // Every load is unconditional (clamped index) and every round first requests all its loads, then calls
    // `hook` (first round only), then converts: the hook is where a one-chunk launch requests its weights.
    auto noop = [](bool) {};
    auto stage = [&](const int k0, const int kc_len, auto&& hook) {
        const int n4 = kc_len >> 2;
        auto ldx = [&](int t, int k4) -> float4 { return ld_act4(a.x + (size_t)t * a.ldx + k0 + k4 * 4); };
        auto ldg = [&](int k4) -> float4 {
            if (!norm) return make_float4(0.f, 0.f, 0.f, 0.f);
            return *(const float4*)(a.gain + k0 + k4 * 4);
        };
        // writes one float4 of row t and returns its sum of squares (for the RMSNorm)
        auto put = [&](int t, int k4, float4 w, const float4& gg) -> float {
            float ss = 0.f;
            if (norm) {
                ss = w.x * w.x + w.y * w.y + w.z * w.z + w.w * w.w;
                w.x *= gg.x; w.y *= gg.y; w.z *= gg.z; w.w *= gg.w;
            }
            if (DT) {
                uint32_t h01, l01, h23, l23;
                split_bf16x2(w.x, w.y, h01, l01);
                split_bf16x2(w.z, w.w, h23, l23);
                *(uint2*)(xs_hi + t * rstride + k4 * 8) = make_uint2(h01, h23);
                *(uint2*)(xs_lo + t * rstride + k4 * 8) = make_uint2(l01, l23);
            } else {
                *(float4*)(xs_hi + t * rstride + k4 * 16) = w;
            }
            return ss;
        };
        if (MG > 0) {
            // x arrives as MG key-split attention partials (no norm in front of an output projection): every piece is
            // sum_s w_s O_s / sum_s w_s L_s with w_s = exp(m_s - max m) of its (row, head).  The normalised weights are
            // worked out once per (row, head) - one pair per thread - and handed over in LDS (the reduction area is
            // free until the MFMAs are done); a piece then costs MG loads and MG multiply-adds.
            constexpr int SP = MG > 0 ? MG : 1;  // (1 only where this branch is dead code)
            constexpr int PMAX = SP == 8 ? 2 : 4;  // pieces per round at most: P * SP float4 loads in flight per thread
            const int total = T * n4;
            const unsigned magic = 0xFFFFFFFFu / (unsigned)n4 + 1u;
            const int npairs = T * a.mg_heads;  // at most the thread count (checked at launch)
            const size_t ml_stride = (size_t)npairs * 2, o_stride = (size_t)T * a.ldx;
            float* wts = (float*)red;  // [npairs][SP]
            const int pr = min(tid, npairs - 1);  // a thread past the end redoes the last pair (same values)
            float m[SP], l[SP];
#pragma unroll
            for (int sp = 0; sp < SP; ++sp) {
                m[sp] = ld_act(a.mg_ml + sp * ml_stride + (size_t)pr * 2);
                l[sp] = ld_act(a.mg_ml + sp * ml_stride + (size_t)pr * 2 + 1);
            }
            auto round = [&](auto np, auto first, int eb, auto&& hk) {
                constexpr int P = decltype(np)::value;
                float4 o[P][SP];
                int tt[P], kk[P];
#pragma unroll
                for (int u = 0; u < P; ++u) {
                    const int e = min(eb + u * nthr, total - 1);
                    tt[u] = (int)__umulhi((unsigned)e, magic);
                    kk[u] = e - tt[u] * n4;
                    const float* op = a.mg_o + (size_t)tt[u] * a.ldx + k0 + kk[u] * 4;
#pragma unroll
                    for (int sp = 0; sp < SP; ++sp) o[u][sp] = ld_act4(op + sp * o_stride);
                }
                hk(true);
                __builtin_amdgcn_sched_barrier(0);  // nothing that uses a loaded value may move above the requests
                if (decltype(first)::value) {
                    float M = -INFINITY;
#pragma unroll
                    for (int sp = 0; sp < SP; ++sp) M = fmaxf(M, m[sp]);
                    float w[SP], L = 0.f;
#pragma unroll
                    for (int sp = 0; sp < SP; ++sp) {
                        w[sp] = (m[sp] == -INFINITY) ? 0.f : expf(m[sp] - M);
                        L += l[sp] * w[sp];
                    }
                    const float inv = 1.f / L;
#pragma unroll
                    for (int sp = 0; sp < SP; ++sp) wts[pr * SP + sp] = w[sp] * inv;
                    __syncthreads();
                }
                // every piece is combined and written, also the clamped duplicates past the end (same value to the same
                // place): the loads above must not become conditional, or the compiler moves them behind the hook
#pragma unroll
                for (int u = 0; u < P; ++u) {
                    const float* wp = wts + (tt[u] * a.mg_heads + (k0 + kk[u] * 4) / a.d_head) * SP;
                    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                    for (int sp = 0; sp < SP; ++sp) {
                        const float w = wp[sp];
                        r.x += o[u][sp].x * w; r.y += o[u][sp].y * w; r.z += o[u][sp].z * w; r.w += o[u][sp].w * w;
                    }
                    put(tt[u], kk[u], r, r);
                }
            };
            // the first round takes as many pieces as the rows need (a padding piece costs SP loads and a conversion)
            if (total <= nthr) {
                round(std::integral_constant<int, 1>{}, std::true_type{}, tid, hook);
            } else if (total <= 2 * nthr || PMAX == 2) {
                round(std::integral_constant<int, 2>{}, std::true_type{}, tid, hook);
                for (int eb = tid + 2 * nthr; eb < total; eb += 2 * nthr)
                    round(std::integral_constant<int, 2>{}, std::false_type{}, eb, noop);
            } else {
                round(std::integral_constant<int, PMAX>{}, std::true_type{}, tid, hook);
                for (int eb = tid + PMAX * nthr; eb < total; eb += PMAX * nthr)
                    round(std::integral_constant<int, PMAX>{}, std::false_type{}, eb, noop);
            }
        } else if (T > 1 && (n4 & 63) == 0) {
            // Several rows whose chunk is a whole number of wavefront-wide pieces: the rows are laid end to
            // end and dealt to all threads, which spreads the conversion work evenly and lets one round of
            // loads (up to 8 per thread, issued together) cover 8 * nthr pieces; 64 consecutive pieces share a row.
            const int total = T * n4;
            const unsigned magic = 0xFFFFFFFFu / (unsigned)n4 + 1u;  // e / n4 == umulhi(e, magic) for e < 2^32 / n4
            // EAGER: every piece is converted and written, also the clamped duplicates past the end (same value to
            // the same place, counted as zero in the sum of squares), so that no load becomes conditional and the
            // compiler cannot move it behind the hook.  Otherwise pieces past the end are skipped.
            auto pieces = [&](auto np, auto eager, int eb, auto&& hk) {
                constexpr int P = decltype(np)::value;
                constexpr bool EAGER = decltype(eager)::value;
                float4 v[P], g[P];
                int tt[P], kk[P];
#pragma unroll
                for (int u = 0; u < P; ++u) {
                    const int e = min(eb + u * nthr, total - 1);
                    tt[u] = (int)__umulhi((unsigned)e, magic);
                    kk[u] = e - tt[u] * n4;
                    v[u] = ldx(tt[u], kk[u]);
                    g[u] = ldg(kk[u]);
                }
                hk(true);
                __builtin_amdgcn_sched_barrier(0);  // the scheduler otherwise pulls the first conversion above the later requests
#pragma unroll
                for (int u = 0; u < P; ++u) {
                    const bool in = eb + u * nthr < total;  // wave-uniform: total and the wave's first piece are multiples of 64
                    if (EAGER || in) {
                        const float ss = put(tt[u], kk[u], v[u], g[u]);
                        if (norm) {
                            const float tot = wave_sum(in ? ss : 0.f);
                            if (lane == 0) ssq[wave * 32 + tt[u]] += tot;
                        }
                    }
                }
            };
            // Up to eight pieces per thread: activations first, weights behind them.  More rows: the conversions are the longer part and a round of eight loads with the
            // weights behind it does not fit the register file, so the weights are requested first and the
            // rounds skip what they do not need.
            if (total <= 2 * nthr) {
                pieces(std::integral_constant<int, 2>{}, std::true_type{}, tid, hook);
            } else if (TCAP > 0 && total <= 3 * nthr) {  // (only in the few-rows kernel: every variant here costs the others)
                pieces(std::integral_constant<int, 3>{}, std::true_type{}, tid, hook);
            } else if (total <= 4 * nthr) {
                pieces(std::integral_constant<int, 4>{}, std::true_type{}, tid, hook);
            } else if (TCAP > 0) {
                // (the few-rows kernel: the launcher guarantees four pieces per thread at most)
            } else if (NT == 1 && total <= 6 * nthr) {  // (above 16 rows the second accumulator set needs the registers)
                pieces(std::integral_constant<int, 6>{}, std::true_type{}, tid, hook);
            } else if (NT == 1 && total <= 8 * nthr) {
                pieces(std::integral_constant<int, 8>{}, std::true_type{}, tid, hook);
            } else {
                hook(false);
                for (int eb = tid; eb < total; eb += nthr * 8)
                    pieces(std::integral_constant<int, 8>{}, std::false_type{}, eb, noop);
            }
        } else {
            // one row, or ragged chunks: few rows - every wave takes a k-slice of every row; otherwise whole
            // rows are dealt to the waves
            auto row = [&](int j, auto&& hk) {
                const int traw = few ? j : wave + NWV * j;
                const bool act = traw < T;  // wave-uniform
                const int t = min(traw, T - 1);
                const int start = few ? tid : lane, step = few ? nthr : 64;
                float ssj = 0.f;
                if (n4 <= step) {  // at most one element per thread (a padding second one would cost a load and a conversion)
                    const int ca = min(start, n4 - 1);
                    const float4 va = ldx(t, ca), ga = ldg(ca);
                    hk(true);
                    __builtin_amdgcn_sched_barrier(0);  // (as above)
                    const float sa = put(t, ca, va, ga);
                    ssj += (act && start < n4) ? sa : 0.f;
                } else if (n4 <= 2 * step) {  // short rows: at most two elements per thread
                    const int ka = start, kb2 = start + step;
                    const int ca = min(ka, n4 - 1), cb = min(kb2, n4 - 1);
                    const float4 va = ldx(t, ca), ga = ldg(ca), vb = ldx(t, cb), gb = ldg(cb);
                    hk(true);
                    __builtin_amdgcn_sched_barrier(0);  // (as above)
                    // unconditional conversions and writes (duplicates carry the same value and count as zero)
                    const float sa = put(t, ca, va, ga), sb = put(t, cb, vb, gb);
                    ssj += (act && ka < n4 ? sa : 0.f) + (act && kb2 < n4 ? sb : 0.f);
                } else {
                    auto rnd = [&](int kb, auto&& hk2) {
                        float4 v[8], g[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u) {  // all loads of the round first
                            const int k4 = min(kb + u * step, n4 - 1);
                            v[u] = ldx(t, k4);
                            g[u] = ldg(k4);
                        }
                        hk2(true);
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            const float su = put(t, min(kb + u * step, n4 - 1), v[u], g[u]);
                            ssj += (act && kb + u * step < n4) ? su : 0.f;
                        }
                    };
                    rnd(start, hk);
                    for (int kb = start + step * 8; kb < n4; kb += step * 8) rnd(kb, noop);
                }
                if (norm && act) {  // this wave's share of sum x^2 of row t, accumulated over the chunks
                    const float tot = wave_sum(ssj);
                    if (lane == 0) ssq[wave * 32 + t] += tot;
                }
            };
            if (ONE) {
                row(0, hook);  // one row: this is the whole staging
            } else {           // ragged widths with several rows (rare): weights first, like the long multi-row case
                hook(false);
                row(0, noop);
            }
            for (int j = 1; j < 8; ++j) {
                if ((few ? j : wave + NWV * j) >= T) break;  // wave-uniform
                row(j, noop);
            }
        }
    };

    const int nkt0 = min(KC, K) / KT;
    if (K <= KC) {
        // ---- one chunk: activations, then both weight buffers, then everything else ----
        // hook(true): both buffers go out behind the activation loads; hook(false) (long staging, which needs the
        // registers): the first buffer goes out ahead of the staging and the second one after it
        // TWO = false (launcher: no wave has more than one batch of tiles): the second buffer does not exist
        bool second_out = false;
        stage(0, K, [&](bool both) {
            request(B0, wkid, nkt0);
            if (TWO && both) request(B1, wkid + S, nkt0);
            second_out = both;
        });
        if (TWO && !second_out) request(B1, wkid + S, nkt0);
        __syncthreads();
        if (!TWO) {
            compute_batch(B0, wkid, nkt0);
        } else {
            for (int kt = wkid;; kt += 2 * S) {
                compute_batch(B0, kt, nkt0);
                if (kt + S >= nkt0) break;
                if (kt + 2 * S < nkt0) request(B0, kt + 2 * S, nkt0);
                compute_batch(B1, kt + S, nkt0);
                if (kt + 2 * S >= nkt0) break;
                if (kt + 3 * S < nkt0) request(B1, kt + 3 * S, nkt0);
            }
        }
    } else if (TCAP == 0) {  // (the few-rows kernel is launched on single-chunk inputs only)
        request(B0, wkid, nkt0);
        for (int k0 = 0; k0 < K; k0 += KC) {
            const int kc_len = min(KC, K - k0);
            if (k0) __syncthreads();  // readers of the previous chunk are done
            stage(k0, kc_len, noop);
            __syncthreads();
            // ---- this wave's weight tiles of the chunk: compute one batch while the next one loads ----
            const int kt_base = k0 / KT, nkt = kc_len / KT;
            const int kn_base = (k0 + KC) / KT, nkt_next = (k0 + KC < K) ? min(KC, K - k0 - KC) / KT : 0;
            // the batch for kt = wkid is already in flight in B0 (kernel entry, or the end of the previous chunk)
            for (int kt = wkid;; kt += 2 * S) {
                {
                    const bool in_chunk = kt + S < nkt;
                    if (in_chunk || nkt_next)
                        request(B1, in_chunk ? kt_base + kt + S : kn_base + wkid, in_chunk ? kt_base + nkt : kn_base + nkt_next);
                    compute_batch(B0, kt, nkt);
                    if (!in_chunk) {  // the next chunk's first batch (if any) went to B1: hand it over
#pragma unroll
                        for (int r = 0; r < RW; ++r)
#pragma unroll
                            for (int u = 0; u < U; ++u) B0[r][u] = B1[r][u];
                        break;
                    }
                }
                {
                    const bool in_chunk = kt + 2 * S < nkt;
                    if (in_chunk || nkt_next)
                        request(B0, in_chunk ? kt_base + kt + 2 * S : kn_base + wkid, in_chunk ? kt_base + nkt : kn_base + nkt_next);
                    compute_batch(B1, kt + S, nkt);
                    if (!in_chunk) break;  // the next chunk's first batch is already in B0
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[r][j] += acc2[r][j];
    // ---- RMSNorm row scales and cross-wave k reduction ----
    if (WK > 1 && !owner) {
#pragma unroll
        for (int r = 0; r < RW; ++r)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                if (j < NT) red[(wave * nacc + r * NT + j) * 64 + lane] = acc[r][j];
    }
    __syncthreads();
    float rsc[2] = {1.f, 1.f};  // 1/rms of this lane's rows
    if (owner) {
        if (norm) {
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                if (nt < NT) {
                    const int t = min(nt * 16 + tok_l, T - 1);
                    float sum = 0.f;
                    for (int w = 0; w < NWV; ++w) sum += ssq[w * 32 + t];
                    rsc[nt] = rsqrtf(sum / (float)K + a.eps);
                }
            }
        }
        if (WK > 1) {
            for (int w2 = 1; w2 < WK; ++w2)
#pragma unroll
                for (int r = 0; r < RW; ++r)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        if (j < NT) acc[r][j] += red[((wave + w2) * nacc + r * NT + j) * 64 + lane];
        }
    }
    // ---- epilogue: lane holds features f = tile*16 + kq*4 + v for row t = nt*16 + tok_l ----
    Stat st[2] = {stat_neutral(), stat_neutral()};
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int t = nt * 16 + tok_l;
        if (nt >= NT || t >= T || !owner) continue;
        const float r = rsc[nt];
        if (RW == 2 && EPI == EPI_ACT) {  // gated FFN: tile0 holds the gate, tile0+1 the linear branch
            if (valid[0] && valid[RW - 1]) {
                const int f0 = (tile0 >> 1) * 16 + kq * 4;
                float o[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float g = acc[0][nt][v] * r, u = acc[RW - 1][nt][v] * r;
                    o[v] = (a.act == BILD_ACT_GATED_GELU ? gelu_tanh_f(g) : silu_f(g)) * u;
                }
                st_act4(a.out + (size_t)t * a.ldo + f0, make_float4(o[0], o[1], o[2], o[3]));
            }
            continue;
        }
#pragma unroll
        for (int rwi = 0; rwi < RW; ++rwi) {
            if (!valid[rwi]) continue;
            const int n0 = (tile0 + rwi) * 16 + kq * 4;
            float v4[4] = {acc[rwi][nt][0] * r, acc[rwi][nt][1] * r, acc[rwi][nt][2] * r, acc[rwi][nt][3] * r};
            switch (epi) {
                case EPI_STORE:
                    st_act4(a.out + (size_t)t * a.ldo + n0, make_float4(v4[0], v4[1], v4[2], v4[3]));
                    break;
                case EPI_RESID: {
                    const float4 o = old[rwi][nt];
                    st_act4(a.out + (size_t)t * a.ldo + n0, make_float4(o.x + v4[0], o.y + v4[1], o.z + v4[2], o.w + v4[3]));
                } break;
                case EPI_ACT:
                    st_act4(a.out + (size_t)t * a.ldo + n0,
                                 make_float4(fmaxf(v4[0], 0.f), fmaxf(v4[1], 0.f), fmaxf(v4[2], 0.f), fmaxf(v4[3], 0.f)));
                    break;
                case EPI_QKV: {
                    const int pos = pos0 + t;
                    const int seg = n0 < a.q_dim ? 0 : (n0 < a.q_dim + a.i_dim ? 1 : 2);
                    const int nn = n0 - (seg == 0 ? 0 : (seg == 1 ? a.q_dim : a.q_dim + a.i_dim));
                    if (rope && seg < 2) {
                        const int hd = nn % a.d_head;
#pragma unroll
                        for (int p2 = 0; p2 < 2; ++p2) {
                            const double fr = exp2(-(double)(hd + 2 * p2) / (double)a.d_head * log2((double)a.rope_base));
                            double sn, cs;
                            sincos((double)pos * fr, &sn, &cs);
                            const float x0 = v4[2 * p2], x1 = v4[2 * p2 + 1];
                            v4[2 * p2] = (float)((double)x0 * cs - (double)x1 * sn);
                            v4[2 * p2 + 1] = (float)((double)x0 * sn + (double)x1 * cs);
                        }
                    }
                    if (seg == 0) {
                        st_act4(a.q_out + (size_t)t * a.i_dim + nn, make_float4(v4[0], v4[1], v4[2], v4[3]));
                    } else if (seg == 1) {  // K: [position][I]
                        const size_t e = (size_t)pos * a.i_dim + nn;
                        if (DT)
                            st_u64((uint16_t*)a.k_cache + e, pack_bf16x2(v4[0], v4[1]), pack_bf16x2(v4[2], v4[3]));
                        else
                            st_act4((float*)a.k_cache + e, make_float4(v4[0], v4[1], v4[2], v4[3]));
                    } else {  // V: transposed, [I][vcap] with the position contiguous
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const size_t e = (size_t)(nn + v) * a.vcap + pos;
                            if (DT)
                                st_u16((uint16_t*)a.v_cache + e, (uint16_t)f2bf(v4[v]));
                            else
                                st_act((float*)a.v_cache + e, v4[v]);
                        }
                    }
                } break;
                case EPI_LMHEAD: {
                    const int row = a.row_off + t;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int n = n0 + v;
                        if (n < a.vocab) {
                            const float z = v4[v] * a.scale;
                            stat_push(st[nt], z, n);
                            if (n == tgt[nt]) a.zt[row] = z;
                            if (a.dbg) a.dbg[(size_t)row * a.vocab + n] = z;
                        }
                    }
                } break;
            }
        }
    }
    if (epi == EPI_LMHEAD) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            st[nt] = stat_merge(st[nt], stat_shfl_xor(st[nt], 16));
            st[nt] = stat_merge(st[nt], stat_shfl_xor(st[nt], 32));
            if (kq == 0) {
                const int t = nt * 16 + tok_l;
                StatPart sp;
                sp.m = st[nt].m; sp.s = st[nt].s; sp.idx = st[nt].idx; sp.pad = 0;
                wstat[wave * 32 + t] = sp;
            }
        }
        __syncthreads();
        if (tid < T) {
            Stat r = stat_neutral();
            for (int w = 0; w < NWV; ++w) {
                const StatPart sp = wstat[w * 32 + tid];
                r = stat_merge(r, Stat{sp.m, sp.s, sp.idx});
            }
            StatPart o;
            o.m = r.m; o.s = r.s; o.idx = r.idx; o.pad = 0;
            a.part[(size_t)vblock * kMaxRows + a.row_off + tid] = o;
        }
    }
}

// SHORT: no wave has more than one batch of tiles - the second weight buffer does not exist (see gemm_row_kernel).
template <int DT, int RW, int EPI, int ROPE, int NT, bool SHORT = false>
__global__ __launch_bounds__(512) void gemm_kernel(const GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    gemm_body<DT, RW, EPI, ROPE, NT, gemm_batch(RW, false, NT), 0, false, !SHORT>(a, (int)blockIdx.x, smem);
}

// The single-row pass (the small model's step, the large model's plain step): the row count is a
// compile-time 1, which removes the multi-row staging paths from the code.
// Padding tiles are not free: a batch slot past the wave's range still costs a load of a clamped tile and, in the
// first buffer, two MFMAs, and on the latency-bound shapes that is most of a wave's instructions (measured on the T5
// pair: 236 -> 206 us per small-model step and 1048 -> 962 us per large-model step once the 512- and 1024-wide inputs
// stopped padding 8 tiles per wave to 24).  VAR picks the batch geometry by the tiles a wave has:
//   1: at most 8   - one batch of 8, no second buffer
//   2: at most 16  - two batches of 8
//   0: more        - batches of 12 (more bytes in flight for the bandwidth-bound shapes)
constexpr int kShortBatch = 8;
template <int DT, int RW, int EPI, int ROPE, int VAR = 0>
__global__ __launch_bounds__(512) void gemm_row_kernel(const GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    gemm_body<DT, RW, EPI, ROPE, 1, VAR ? kShortBatch / RW : gemm_batch(RW, true), 0, true, VAR != 1>(a, (int)blockIdx.x, smem);
}

// Two to four rows (the bulk of the large model's review passes) on a single-chunk input: the same body without the
// staging rounds for more rows and without the multi-chunk loop.  Run through the general kernel a pass of these row
// counts costs about 0.7 us more per projection (measured: one row through gemm_kernel 1018 us per T5-large pass,
// through gemm_row_kernel 911 us), which is code size and register pressure, not work.
template <int DT, int RW, int EPI, int ROPE, bool SHORT>
__global__ __launch_bounds__(512) void gemm_few_kernel(const GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    gemm_body<DT, RW, EPI, ROPE, 1, gemm_batch(RW, false, 1), 0, false, !SHORT, 4>(a, (int)blockIdx.x, smem);
}

// Output projection whose input is still in key-split attention partials (merged while staging).
template <int DT, int SPLITS, bool SHORT = false>
__global__ __launch_bounds__(512) void gemm_merge_kernel(const GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    gemm_body<DT, 1, EPI_RESID, 0, 1, gemm_batch(1, false), SPLITS, false, !SHORT>(a, (int)blockIdx.x, smem);
}

// Between kMaxRows and kDenseMinRows rows (an encoder over a source of a few hundred tokens): blockIdx.y picks a block
// of kMaxRows rows and the same body runs on it.  The blocks of one feature group re-read its weight tiles, which by
// then sit in L2 or the memory-side cache, so HBM still streams every weight about once.  At these sizes a projection
// is a GFLOP or two: too little to fill the dense-tile kernel's 64-row tiles on 256 compute units (measured on 512 rows
// of 1024..4096-wide projections: 12..40 us per launch there, 12..25 us here); longer passes go to gemm_dense.hip.
template <int DT, int RW, int EPI, int ROPE>
__global__ __launch_bounds__(512) void gemm_rows_kernel(const GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
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
    const int nch = (a.W.k + kc_max - 1) / kc_max;
    const int kc = ((a.W.k + nch - 1) / nch + kt - 1) / kt * kt;
    a.kc = kc;
    const int tiles_last = (a.W.k - (nch - 1) * kc) / kt;
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
    while (wk_lat < 8 && a.W.tk / wk_lat > batch) wk_lat *= 2;
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
        a.wk = std::max(1, std::min(8 / wr, tiles_chunk));
        a.nwv = a.wk * wr;
        return;
    }
    // feature groups: as many as keep >= 512 workgroups; at least 4 waves per workgroup, 8 once a thread of a 4-wave
    // workgroup would stage more than eight pieces (staging the activations is then the longer part, and it is shared
    // by all waves; measured on 24 layers of 1024-wide projections: 4 waves win up to 8 rows, 1365 against 1490 us per
    // pass, 8 waves from 9 rows, 1505 against 1578)
    int wr = std::max(1, ((long)a.T * a.W.k > 8192 && a.epi != EPI_LMHEAD ? 8 : 4) / wk);
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
    (const void*)gemm_row_kernel<DTV, 1, EPI_STORE, 0, 2>, (const void*)gemm_row_kernel<DTV, 1, EPI_RESID, 0, 2>, \
    (const void*)gemm_row_kernel<DTV, 1, EPI_QKV, 0, 2>, (const void*)gemm_row_kernel<DTV, 1, EPI_QKV, 1, 2>, \
    (const void*)gemm_row_kernel<DTV, 1, EPI_ACT, 0, 2>, \
    (const void*)gemm_row_kernel<DTV, 2, EPI_ACT, 0, 1>, (const void*)gemm_row_kernel<DTV, 2, EPI_ACT, 0, 2>, \
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
    return attention_init();
}

hipError_t launch_gemm(const GemmArgs& a, int dtype, hipStream_t st) {
    if (hipError_t e = raise_lds_limits(); e != hipSuccess) return e;
    if (a.T >= kDenseMinRows) return launch_gemm_dense(a, dtype, st);
    const size_t smem = gemm_lds_bytes(a, dtype);
    const unsigned row_blocks = (unsigned)((a.T + kMaxRows - 1) / kMaxRows);
    if (row_blocks > 1 && a.epi == EPI_LMHEAD) return hipErrorInvalidValue;  // softmax partials are per pass
    if ((a.gain != nullptr) != (a.epi != EPI_RESID)) return hipErrorInvalidValue;  // the kernels fix the norm by the epilogue
    if (a.mg_splits > 1) {
        // merged staging: 2, 4 or 8 splits, up to 16 rows, one (row, head) pair per thread, weights in the reduction area
        const int sp = a.mg_splits, npairs = a.T * a.mg_heads;
        if ((sp != 2 && sp != 4 && sp != 8) || a.gain || a.T > 16 || a.epi != EPI_RESID || a.rw != 1 || a.mg_heads < 1 ||
            npairs > 64 * a.nwv || (size_t)npairs * sp * 4 > (size_t)gemm_red_bytes(a.nwv, 1))
            return hipErrorInvalidValue;
        const dim3 grid1((unsigned)gemm_num_blocks(a)), block1(64 * a.nwv);
#define BILD_MG(DTV, SH)                                                                       \
    do {                                                                                        \
        if (sp == 2) hipLaunchKernelGGL((gemm_merge_kernel<DTV, 2, SH>), grid1, block1, smem, st, a); \
        else if (sp == 4) hipLaunchKernelGGL((gemm_merge_kernel<DTV, 4, SH>), grid1, block1, smem, st, a); \
        else hipLaunchKernelGGL((gemm_merge_kernel<DTV, 8, SH>), grid1, block1, smem, st, a);   \
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
            hipLaunchKernelGGL((gemm_rows_kernel<DTV, RWV, EPIV, ROPEV>), grid, block, smem, st, a); \
        else if (a.T == 1 && RWV == 2 && one_chunk && per_wave <= kShortBatch / 2)                  \
            hipLaunchKernelGGL((gemm_row_kernel<DTV, 2, EPI_ACT, 0, 1>), grid, block, smem, st, a); \
        else if (a.T == 1 && RWV == 2 && one_chunk && (per_wave <= kShortBatch || (per_wave % 4 == 0 && per_wave % 6 != 0))) \
            hipLaunchKernelGGL((gemm_row_kernel<DTV, 2, EPI_ACT, 0, 2>), grid, block, smem, st, a); \
        else if (a.T == 1 && RWV == 1 && one_chunk && per_wave <= kShortBatch)                      \
            hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPIV, ROPEV, 1>), grid, block, smem, st, a); \
        else if (a.T == 1 && RWV == 1 && one_chunk && (per_wave <= 2 * kShortBatch || (per_wave % kShortBatch == 0 && per_wave % 12 != 0))) \
            hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPIV, ROPEV, 2>), grid, block, smem, st, a); \
        else if (a.T == 1)                                                                          \
            hipLaunchKernelGGL((gemm_row_kernel<DTV, RWV, EPIV, ROPEV>), grid, block, smem, st, a); \
        else if (a.T > 16)                                                                          \
            hipLaunchKernelGGL((gemm_kernel<DTV, RWV, EPIV, ROPEV, 2>), grid, block, smem, st, a);  \
        else if (RWV == 1 && few_ok && per_wave <= gemm_batch(1, false))                            \
            hipLaunchKernelGGL((gemm_few_kernel<DTV, 1, EPIV, ROPEV, true>), grid, block, smem, st, a); \
        else if (RWV == 1 && few_ok)                                                                \
            hipLaunchKernelGGL((gemm_few_kernel<DTV, 1, EPIV, ROPEV, false>), grid, block, smem, st, a); \
        else if (RWV == 1 && one_chunk && per_wave <= gemm_batch(1, false))                         \
            hipLaunchKernelGGL((gemm_kernel<DTV, 1, EPIV, ROPEV, 1, true>), grid, block, smem, st, a); \
        else                                                                                        \
            hipLaunchKernelGGL((gemm_kernel<DTV, RWV, EPIV, ROPEV, 1>), grid, block, smem, st, a);  \
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
            if (a.rw == 4 && a.T == 1)                                           \
                hipLaunchKernelGGL((gemm_row_kernel<DTV, 4, EPI_LMHEAD, 0>), grid, block, smem, st, a); \
            else if (a.rw == 4 && a.T <= 16)                                     \
                hipLaunchKernelGGL((gemm_kernel<DTV, 4, EPI_LMHEAD, 0, 1>), grid, block, smem, st, a); \
            else if (a.rw != 1)                                                  \
                return hipErrorInvalidValue;                                     \
            else if (a.T == 1 && one_chunk && per_wave <= 32 && per_wave % kShortBatch == 0) /* batches of 8 fit exactly */ \
                hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPI_LMHEAD, 0, 2>), grid, block, smem, st, a); \
            else if (a.T == 1)                                                   \
                hipLaunchKernelGGL((gemm_row_kernel<DTV, 1, EPI_LMHEAD, 0>), grid, block, smem, st, a); \
            else if (a.T > 16)                                                   \
                hipLaunchKernelGGL((gemm_kernel<DTV, 1, EPI_LMHEAD, 0, 2>), grid, block, smem, st, a); \
            else                                                                 \
                hipLaunchKernelGGL((gemm_kernel<DTV, 1, EPI_LMHEAD, 0, 1>), grid, block, smem, st, a); \
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
    for (int k = threadIdx.x; k < a.d; k += blockDim.x) {
        const size_t tile = (size_t)(row >> 4) * a.E.tk + (k / KT);
        const int ln = (row & 15) + 16 * ((k % KT) / PL), j = k % PL;
        const char* p = (const char*)a.E.w + tile * kTileBytes + ln * 16;
        float v = DT ? bf2f(((const uint16_t*)p)[j]) : ((const float*)p)[j];
        v *= a.embed_scale;
        if (a.sinusoidal) {
            const double ang = (double)pos * exp2(-(double)(2 * (k >> 1)) / (double)a.d * lg);
            v += (float)((k & 1) ? cos(ang) : sin(ang));
        }
        st_act(a.x + (size_t)t * a.d + k, v);
    }
}

template <int DT>
__global__ __launch_bounds__(256) void embed_kernel(const EmbedArgs a) { embed_body<DT>(a, (int)blockIdx.x); }

hipError_t launch_embed(const EmbedArgs& a, int dtype, hipStream_t st) {
    if (dtype)
        hipLaunchKernelGGL(embed_kernel<1>, dim3(a.T), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(embed_kernel<0>, dim3(a.T), dim3(256), 0, st, a);
    return hipGetLastError();
}


// =====================================================================================
// Merge of the LM-head partials + policy + commit.  One workgroup.
//   mode 0  small step: token = argmax, fallback iff max p < alpha or n_max drafts pending
//   mode 1  review: nll_i = lse_i - z_i[draft_i]; r = first i with nll_i > alpha, else n;
//           y <- y[:draft_start + r] + [argmax of row r]; cache lengths follow
//   mode 2  plain greedy: always append
//   mode 3  no LM head: only advance the cache length by the rows consumed
//   mode 4  measurement: merge the statistics, commit nothing
// =====================================================================================
// LDS use of finish_body (from the start of the workgroup's LDS)
constexpr int kFinishLds = 3 * kMaxRows * 4;
// LDS of the sampling variant behind that: 16 waves x 16 bins, 1024 per-thread masses, a few scalars
constexpr int kDrawLds = 16 * 16 * 4 + 1024 * 4 + 128;

// Order-preserving integer image of a float: a < b  <=>  key(a) < key(b).
__device__ __forceinline__ uint32_t float_key(float f) {
    const uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Nucleus draw of the sampling variant (Appendix, BiLD with Sampling), by the whole workgroup (at most
// 1024 threads).  Nucleus = every token whose probability is at least that of the least likely member of
// the smallest top set reaching top_p; the draw walks the members in increasing id until their running mass
// exceeds u * mass.  The threshold is found exactly, as an integer key, by a radix search of 4 bits per
// sweep over the logits: with e_i = exp(z_i - m), K is the largest key with sum_{key_i >= K} e_i >= top_p * sum e_i.
// Returns the token to every thread.  `ws` is kDrawLds bytes of LDS.
__device__ __forceinline__ int nucleus_draw(const float* __restrict__ z, int V, float m, float top_p, float u, char* ws) {
    float* bins = (float*)ws;              // [16 waves][16]
    float* tmass = bins + 16 * 16;         // [1024]
    float* sc = tmass + 1024;              // scalars
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nthr = blockDim.x, nwv = nthr >> 6;
    uint32_t K = 0;
    float target = 0.f, mass = 0.f;
    // A row of up to 32 logits per thread stays in registers for all sweeps (one batch of loads); longer rows
    // are re-read from L2 every sweep, eight loads at a time.
    constexpr int CACHED = 32;
    const bool cached = V <= CACHED * nthr;
    float zc[CACHED];
    if (cached) {
#pragma unroll
        for (int c = 0; c < CACHED; ++c) {
            const int i = tid + c * nthr;
            zc[c] = i < V ? z[i] : -INFINITY;  // -inf: weight exp(-inf) = 0 and the lowest key
        }
    }
    for (int shift = 28; shift >= 0; shift -= 4) {
        float h[16], sure = 0.f;  // sure: members of every candidate of this sweep (their key is 16 steps or more above K)
#pragma unroll
        for (int j = 0; j < 16; ++j) h[j] = 0.f;
        auto take = [&](float zi) {
            const uint32_t k = float_key(zi);
            if (k >= K) {  // below K: excluded for good; the set still in play shrinks with every sweep
                const uint32_t q = (k - K) >> shift;
                const float e = expf(zi - m);
                if (q >= 16u) {
                    sure += e;
                } else {
#pragma unroll
                    for (int j = 0; j < 16; ++j) h[j] += (q == (uint32_t)j) ? e : 0.f;
                }
            }
        };
        if (cached) {
#pragma unroll
            for (int c = 0; c < CACHED; ++c) take(zc[c]);
        } else {
            for (int i0 = tid; i0 < V; i0 += nthr * 8) {
                float v[8];
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    const int i = i0 + c * nthr;
                    v[c] = i < V ? z[i] : -INFINITY;
                }
#pragma unroll
                for (int c = 0; c < 8; ++c) take(v[c]);
            }
        }
        h[15] += sure;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float t = wave_sum(h[j]);
            if (lane == 0) bins[wave * 16 + j] = t;
        }
        __syncthreads();
        if (tid < 16) {  // bin totals over the waves, one bin per thread
            float t = 0.f;
            for (int w = 0; w < nwv; ++w) t += bins[w * 16 + tid];
            sc[8 + tid] = t;
        }
        __syncthreads();
        if (tid == 0) {
            if (shift == 28) {
                float all = 0.f;
                for (int j = 0; j < 16; ++j) all += sc[8 + j];
                sc[2] = top_p * all;
            }
            const float tgt = sc[2];
            float above = 0.f;  // mass of the members of candidate j = sum of bins j..15
            int pick = 0;
            float pick_mass = 0.f;
            for (int j = 15; j >= 0; --j) {
                above += sc[8 + j];
                if (j == 0 || above >= tgt) {
                    pick = j;
                    pick_mass = above;
                    break;
                }
            }
            sc[0] = __uint_as_float((uint32_t)pick);
            sc[1] = pick_mass;
        }
        __syncthreads();
        K += __float_as_uint(sc[0]) << shift;
        mass = sc[1];
        target = sc[2];
        __syncthreads();
    }
    (void)target;
    // ---- the draw: every thread owns a run of consecutive ids ----
    const int chunk = (V + nthr - 1) / nthr;
    const int i0 = min(tid * chunk, V), i1 = min(i0 + chunk, V);
    float mine = 0.f;
    for (int i = i0; i < i1; ++i) {
        const float zi = z[i];
        if (float_key(zi) >= K) mine += expf(zi - m);
    }
    tmass[tid] = mine;
    const float wsum = wave_sum(mine);
    if (lane == 0) bins[wave] = wsum;
    __syncthreads();
    if (tid == 0) {
        const float t = u * mass;
        float run = 0.f;
        int w = 0;
        for (; w < nwv - 1; ++w) {  // the wave whose ids hold the target mass
            if (run + bins[w] > t) break;
            run += bins[w];
        }
        int th = w * 64;
        const int th_end = w * 64 + 63;
        for (; th < th_end; ++th) {
            if (run + tmass[th] > t) break;
            run += tmass[th];
        }
        sc[3] = __uint_as_float((uint32_t)th);
        sc[4] = run;
        sc[5] = t;
        sc[6] = __uint_as_float(0xFFFFFFFFu);
    }
    __syncthreads();
    const int owner = (int)__float_as_uint(sc[3]);
    if (tid == owner) {
        float run = sc[4];
        const float t = sc[5];
        int tok = -1, last = -1;
        for (int i = i0; i < i1; ++i) {
            const float zi = z[i];
            if (float_key(zi) >= K) {
                last = i;
                run += expf(zi - m);
                if (run > t) {
                    tok = i;
                    break;
                }
            }
        }
        sc[6] = __uint_as_float((uint32_t)(tok >= 0 ? tok : last));
    }
    __syncthreads();
    int tok = (int)__float_as_uint(sc[6]);
    if (tok < 0) {  // rounding left the target beyond the last member: take the highest member id
        int best = -1;
        for (int i = tid; i < V; i += nthr)
            if (float_key(z[i]) >= K) best = max(best, i);
        for (int o = 32; o > 0; o >>= 1) best = max(best, __shfl_xor(best, o, 64));
        if (lane == 0) bins[wave] = __int_as_float(best);
        __syncthreads();
        for (int w = 0; w < nwv; ++w) tok = max(tok, __float_as_int(bins[w]));
    }
    return tok;
}

template <bool SAMPLE>
__device__ __forceinline__ void finish_body(const FinishArgs& a, char* lds) {
    float* rm = (float*)lds;
    float* rsum = rm + kMaxRows;
    int* ridx = (int*)(rsum + kMaxRows);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nthr = blockDim.x, nwv = nthr >> 6;
    Ctl* c = a.ctl;
    // the control words the policy needs, requested now (nothing in this kernel writes them before they are used): their
    // trip from memory overlaps with the partials' instead of following it
    const int c_ylen = c->y_len, c_ds = c->draft_start, c_nmax = c->n_max, c_len0 = c->len[0], c_lenw = c->len[a.which];
    const float c_afb = c->alpha_fb, c_arb = c->alpha_rb;
    const int c_seq = c->seq;
    if (a.mode != 3) {
        // rows are dealt to the waves; a wave's lanes share the partials of its row (eight loads in flight
        // per lane), so the rows of a review merge side by side and a single row costs one round trip
        for (int t = wave; t < a.T; t += nwv) {
            Stat r = stat_neutral();
            for (int p0 = lane; p0 < a.nparts; p0 += 64 * 8) {
                StatPart sp[8];
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    sp[k] = a.part[(size_t)min(p0 + k * 64, a.nparts - 1) * kMaxRows + a.row_off + t];
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    if (p0 + k * 64 < a.nparts) r = stat_merge(r, Stat{sp[k].m, sp[k].s, sp[k].idx});
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) r = stat_merge(r, stat_shfl_xor(r, o));
            if (lane == 0) {
                rm[t] = r.m;
                rsum[t] = r.s;
                ridx[t] = r.idx;
            }
        }
        __syncthreads();
    }
    // Sampling variant: the token that will be committed is drawn by the whole workgroup from the row the
    // policy selects (the last row of a step; row r of a review), at the position it will occupy.
    int drawn = -1;
    if (SAMPLE && a.top_p > 0.f && a.mode <= 2) {
        int* sel = (int*)(lds + kFinishLds);  // [0] row, [1] position
        if (tid == 0) {
            int row = a.T - 1, pos = c_ylen;
            if (a.mode == 1) {
                const int n = a.T - 1;
                const float alpha = c_arb;
                row = n;
                for (int i = 0; i < n; ++i)
                    if ((rm[i] + logf(rsum[i])) - a.zt[a.row_off + i] > alpha) {
                        row = i;
                        break;
                    }
                pos = c_ds + row;
            }
            sel[0] = row;
            sel[1] = pos;
        }
        __syncthreads();
        const int row = sel[0], pos = sel[1];
        drawn = nucleus_draw(a.logits + (size_t)(a.row_off + row) * a.vocab, a.vocab, rm[row], a.top_p, a.u[pos],
                             lds + kFinishLds + 16);
    }
    if (tid == 0) {
        const int w = a.which;
        const int y_len = c_ylen, ds = c_ds, n_max = c_nmax;
        if (a.mode == 3) {
            c->len[w] = c_lenw + a.rows_consumed;
        } else {
            for (int t = 0; t < a.T; ++t) c->res_rowtok[t] = ridx[t];
            if (a.mode == 0 || a.mode == 2) {
                const int tok = drawn >= 0 ? drawn : ridx[a.T - 1];
                const float pmax = 1.f / rsum[a.T - 1];
                const bool low = (a.mode == 0) && (pmax < c_afb);
                const bool forced = (a.mode == 0) && n_max > 0 && (y_len - ds) >= n_max;
                const bool fb = low || forced;
                c->len[w] = c_lenw + a.rows_consumed;
                if (!fb && y_len < a.y_cap) {
                    a.y[y_len] = tok;
                    c->y_len = y_len + 1;
                    if (a.mode == 2) c->draft_start = y_len + 1;
                }
                c->res_tok = tok;
                c->res_flag = (fb ? 1 : 0) | ((forced && !low) ? 2 : 0);
                c->res_pmax = pmax;
            } else if (a.mode == 1) {  // review of n = T - 1 drafts
                const int n = a.T - 1;
                const float alpha = c_arb;
                int r = n;
                for (int i = 0; i < n; ++i) {
                    const float nll = (rm[i] + logf(rsum[i])) - a.zt[a.row_off + i];
                    c->res_nll[i] = nll;
                    if (r == n && nll > alpha) r = i;
                }
                const int tok = drawn >= 0 ? drawn : ridx[r];
                a.y[ds + r] = tok;
                c->y_len = ds + r + 1;
                c->len[1] = ds + r;
                c->len[0] = min(c_len0, ds + r);
                c->draft_start = ds + r + 1;
                c->res_r = r;
                c->res_n = n;
                c->res_tok = tok;
                c->res_pmax = 1.f / rsum[r];
                c->res_flag = 0;
            }
        }
        __threadfence();
    }
    __syncthreads();
    // mirror the control block into pinned host memory for the caller; the pass counter goes last, behind a
    // system-wide fence, so that a host that sees the new count also sees every other word
    if (a.host_mirror) {
        static_assert(offsetof(Ctl, seq) == sizeof(Ctl) - 4, "seq must be the last word of the control block");
        const int words = sizeof(Ctl) / 4 - 1;
        for (int i = tid; i < words; i += nthr)
            ((volatile int*)a.host_mirror)[i] = __hip_atomic_load((int*)c + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __threadfence_system();
        __syncthreads();
        if (tid == 0) {
            const int sq = c_seq + 1;
            c->seq = sq;
            ((volatile int*)a.host_mirror)[words] = sq;
        }
    }
}

__global__ __launch_bounds__(256) void finish_kernel(const FinishArgs a) {
    __shared__ __attribute__((aligned(16))) char lds[kFinishLds];
    finish_body<false>(a, lds);
}

__global__ __launch_bounds__(1024) void finish_sample_kernel(const FinishArgs a) {
    __shared__ __attribute__((aligned(16))) char lds[kFinishLds + 16 + kDrawLds];
    finish_body<true>(a, lds);
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

hipError_t launch_finish(const FinishArgs& a, hipStream_t st) {
    if (a.top_p > 0.f && a.mode <= 2) {
        if (!a.logits || !a.u || a.vocab < 1) return hipErrorInvalidValue;
        hipLaunchKernelGGL(finish_sample_kernel, dim3(1), dim3(1024), 0, st, a);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(256), 0, st, a);
    return hipGetLastError();
}


}  // namespace bild
