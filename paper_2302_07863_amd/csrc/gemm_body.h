// Body of the weight-streaming skinny GEMM of the BiLD decoding path (gfx950), shared by the translation units that
// instantiate its launch wrappers (kernels.hip: fp32 activations in; gemm_pre.hip: activations handed over already
// split into bf16 planes by the producing kernel).
#pragma once
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

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Hot arguments.  The kernels take their arguments as one structure, which the wavefronts fetch from memory when they
// start: a round trip before the first address can be formed, and a second one where the compiler fetches a field
// only in front of its first use.  The few values the first requests depend on - where the weights and the activations
// are, how the workgroup is cut into waves - are therefore passed a second time as leading scalar parameters, which
// gfx950 delivers in scalar registers at wave start (kernel-argument preload: the library is compiled with it
// on); the structure behind them is read for everything else while those requests are on their way.
//   h_w             weight tiles (W.w)
//   h_x, h_g        activations and norm gain (x, gain) | input planes (xb_hi, xb_lo) | key-split partials (mg_o, mg_ml)
//   h_px            partial results a reader adds (px; their stride is kMaxRows * ldx)
//   h_tn, h_tk      W.tn, W.tk (W.k is tk whole tiles)
//   h_geom          wk | log2(wk) << 4 | nwv << 8 | T << 12
//   h_kc, h_ldx     kc, ldx
//   h_aux           readers of partial results: x_out - x in floats | key-split partials: mg_heads | d_head << 16
#define BILD_GEMM_HOT_PARAMS                                                                                      \
    const void* __restrict__ h_w, const void* __restrict__ h_x, const void* __restrict__ h_g,                     \
        const float* __restrict__ h_px, const int h_tn, const int h_tk, const int h_geom, const int h_kc,         \
        const int h_ldx, const int h_aux
#define BILD_GEMM_HOT_NAMES h_w, h_x, h_g, h_px, h_tn, h_tk, h_geom, h_kc, h_ldx, h_aux
enum HotKind : int { HOT_X = 0, HOT_PRE = 1, HOT_MG = 2 };
template <int KIND, int DT>
__device__ __forceinline__ GemmArgs gemm_hot(const GemmArgs& a, BILD_GEMM_HOT_PARAMS) {
    GemmArgs b = a;
    b.W.w = h_w; b.W.k = h_tk * (DT ? 32 : 16); b.W.tn = h_tn; b.W.tk = h_tk;
    b.wk = h_geom & 15; b.lwk = (h_geom >> 4) & 15; b.nwv = (h_geom >> 8) & 15; b.T = h_geom >> 12;
    b.kc = h_kc; b.ldx = h_ldx;
    if (KIND == HOT_X) {
        b.x = (const float*)h_x; b.gain = (const float*)h_g; b.px = h_px; b.px_stride = (int64_t)kMaxRows * h_ldx;
        b.x_out = const_cast<float*>((const float*)h_x) + h_aux;
    }
    if (KIND == HOT_PRE) { b.xb_hi = (const uint16_t*)h_x; b.xb_lo = (const uint16_t*)h_g; }
    if (KIND == HOT_MG) { b.mg_o = (const float*)h_x; b.mg_ml = (const float*)h_g; b.mg_heads = h_aux & 0xFFFF; b.d_head = h_aux >> 16; }
    return b;
}

// Four consecutive features of row t, handed to the next projection as high and low bf16 parts.
__device__ __forceinline__ void put_planes(const GemmArgs& a, int t, int n0, const float (&w)[4]) {
    uint32_t h01, l01, h23, l23;
    split_bf16x2(w[0], w[1], h01, l01);
    split_bf16x2(w[2], w[3], h23, l23);
    const size_t off = (size_t)t * a.nx_ld + n0;
    st_u64(a.nx_hi + off, h01, h23);
    st_u64(a.nx_lo + off, l01, l23);
}

// `vblock` is the index of the feature-tile group this workgroup handles (blockIdx.x); `smem` is its dynamic LDS.
// KS: this workgroup covers only a slice of the inputs (a.k_len inputs from tile a.k_off_tiles on; a.x points at the
// slice): the launch wrapper gives every slice its own output (EPI_PART), and the projection that reads the result adds the
// slices up while staging.  PS > 0: that reader - its input is a.x plus PS partial results a.px[j] (fixed order; a producer with fewer leaves the
// rest of the PS slots zero), and the
// workgroup with index 0 also writes the sum to a.x_out (another buffer than a.x, which the other workgroups still read).
// EMB (single-row launches on one chunk): the input row is gathered from the embedding matrix (GemmArgs::e_w ..), so the
// pass needs no embedding kernel in front of its first projection; workgroup 0 writes the row to a.x_out for the residual adds.
// EX (single-batch launches, TWO = false): every wave has exactly U input tiles - no tile index is clamped and no product
// is cancelled, which takes four scalar instructions out of the way of each weight request (the last request of a wave then
// goes out some 0.1 us earlier, and the stage ends that much earlier).
// PRE: the input arrives as high / low bf16 planes with the consumer's norm gain already applied, written by the
// kernel that produced it (a.xb_hi, a.xb_lo; a.ssq_part holds that kernel's per-wave sums of squares): staging is a
// plain copy into LDS.  NX: this kernel's epilogue hands its own output on in that form (a.nx_*).
template <int DT, int RW, int EPI, int ROPE, int NT, int U = gemm_batch(RW, false, NT), int MG = 0,
          bool ONE = false, bool TWO = true, int TCAP = 0, bool PRE = false, bool NX = false, int PS = 0, bool KS = false,
          bool EMB = false, bool EX = false>
__device__ __forceinline__ void gemm_body(const GemmArgs& a, const int vblock, char* smem) {
    constexpr int KT = DT ? 32 : 16;
    // the wave index through readfirstlane: the compiler then knows that it - and every tile index, weight address and
    // range test derived from it - is the same in all lanes, and keeps them in scalar registers
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int NWV = a.nwv, nthr = NWV << 6;  // (the launch has 64 * nwv threads; blockDim would be one more fetch)
    const int T = ONE ? 1 : a.T, K = KS ? a.k_len : a.W.k, KC = a.kc;
    const int WK = a.wk, WR = NWV >> a.lwk;  // wk is a power of two
    const int wkid = wave & (WK - 1), wrid = wave >> a.lwk;
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
    constexpr bool norm = EPI != EPI_RESID && EPI != EPI_PART;
    const bool few = T < 4;  // few rows: all waves share each row and split it along k
    const bool owner = (wkid == 0);
    bool valid[RW];
    const char* wbase[RW];
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        valid[r] = tile0 + r < a.W.tn;
        wbase[r] = (const char*)a.W.w + ((size_t)min(tile0 + r, a.W.tn - 1) * a.W.tk + (KS ? a.k_off_tiles : 0)) * kTileBytes;  // scalar; the lane part is added per load
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
            const int ktc = EX ? kt_abs + u * WK : min(kt_abs + u * WK, kt_end - 1);
#pragma unroll
            for (int r = 0; r < RW; ++r) B[r][u] = *(const uint4*)(wbase[r] + (size_t)ktc * kTileBytes + lane16);
        }
    };

    // What only the epilogue needs - the residual values, the position of row 0, the target ids - is requested by
    // `late`, which runs right behind the first weight requests: the fields of the argument structure it reads (and the
    // position behind a pointer in it) are two more trips to memory, and nothing in front of the first requests
    // may wait for them.  The residual loads are unconditional loads from clamped addresses (a conditional load would
    // have to be waited for where the branches join).
    float4 old[RW][2];
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) old[r][nt] = make_float4(0.f, 0.f, 0.f, 0.f);
    int pos0 = 0;
    int tgt[2] = {-1, -1};
    auto late = [&]() {
        if (lane < 32) ssq[wave * 32 + lane] = 0.f;  // each wave owns (and later accumulates into) its own row
        if (tid < 4) ((uint4*)zblk)[tid] = make_uint4(0u, 0u, 0u, 0u);
        if (epi == EPI_RESID) {
#pragma unroll
            for (int r = 0; r < RW; ++r)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    old[r][nt] = ld_act4(a.out + (size_t)min(nt * 16 + tok_l, T - 1) * a.ldo + min(tile0 + r, a.W.tn - 1) * 16 + kq * 4);
        }
        if (epi == EPI_QKV || epi == EPI_LMHEAD) pos0 = (a.pos_ptr ? *a.pos_ptr : 0) + a.pos_add;
        if (epi == EPI_LMHEAD) {
            const int ylen = *a.ylen_ptr;
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                const int ti = pos0 + nt * 16 + tok_l + 1;
                if (nt * 16 + tok_l < T && ti < ylen) tgt[nt] = a.y[ti];
            }
        }
    };

    // PRE: the sums of squares of the rows come from the producer, one partial per wave of it that owned output tiles.
    // Wave w adds the partials of rows w, w + NWV, ...: they are requested behind the weights (ssq_request) and added
    // after the products (ssq_reduce), when whatever was requested before them has arrived anyway.
    constexpr int SSL = NT == 2 ? 8 : 4;  // rows per wave at most (launcher: T <= SSL * NWV)
    constexpr int SSC = 4;                // 64 partials per load round: at most 256 partials
    float sv[SSL][SSC];
    auto ssq_request = [&]() {
#pragma unroll
        for (int j = 0; j < SSL; ++j) {
            const int t = wave + NWV * j;  // wave-uniform
#pragma unroll
            for (int c = 0; c < SSC; ++c) {
                sv[j][c] = 0.f;
                if (t < T && c * 64 < a.ssq_parts)
                    sv[j][c] = ld_act(a.ssq_part + (size_t)min(lane + c * 64, a.ssq_parts - 1) * kMaxRows + t);
            }
        }
    };
    auto ssq_reduce = [&]() {
#pragma unroll
        for (int j = 0; j < SSL; ++j) {
            const int t = wave + NWV * j;
            if (t < T) {
                float sum = 0.f;
#pragma unroll
                for (int c = 0; c < SSC; ++c) sum += (lane + c * 64 < a.ssq_parts) ? sv[j][c] : 0.f;
                const float tot = wave_sum(sum);
                if (lane == 0) ssq[wave * 32 + t] = tot;
            }
        }
    };

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
            compute(At, kt + u * WK, EX || kt + u * WK < nkt);
        }
    };

    // ---- stage x[:, k0 : k0+kc_len] (times the norm gain) into LDS ----
    // Every load is unconditional (clamped index) and every round first requests all its loads, then calls
    // `hook` (first round only), then converts: the hook is where a one-chunk launch requests its weights.
    auto noop = [](bool) {};
    auto stage = [&](const int k0, const int kc_len, auto&& hook) {
        const int n4 = kc_len >> 2;
        struct XV { float4 p[PS + 1]; };  // one piece of x: the base and the PS partial results still to be added
        auto ldx = [&](int t, int k4) -> XV {
            XV r;
            const size_t off = (size_t)t * a.ldx + k0 + k4 * 4;
            r.p[0] = ld_act4(a.x + off);
#pragma unroll
            for (int j = 0; j < PS; ++j) r.p[j + 1] = ld_act4(a.px + (size_t)j * a.px_stride + off);
            return r;
        };
        auto ldg = [&](int k4) -> float4 {
            if (!norm) return make_float4(0.f, 0.f, 0.f, 0.f);
            return *(const float4*)(a.gain + k0 + k4 * 4);
        };
        // writes one float4 of row t and returns its sum of squares (for the RMSNorm)
        auto put = [&](int t, int k4, const XV& wv, const float4& gg) -> float {
            float4 w = wv.p[0];
#pragma unroll
            for (int j = 0; j < PS; ++j) { w.x += wv.p[j + 1].x; w.y += wv.p[j + 1].y; w.z += wv.p[j + 1].z; w.w += wv.p[j + 1].w; }
            if ((PS > 0 || EMB) && vblock == 0) st_act4(a.x_out + (size_t)t * a.ldx + k0 + k4 * 4, w);  // the residual stream, for later readers
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
        if constexpr (EMB) {
            // The weights go out first: the row's address is behind two dependent scalar loads (position, token id), so
            // the gather is a third trip, and the weights' own trip covers most of the chain.  Pieces in pairs (clamped
            // duplicates carry the same value to the same place and count as zero in the sum of squares).
            hook(true);
            const int base = *a.e_base_ptr + a.e_base_add;
            const int tok = a.e_tokens[base];
            int erow_i = tok + a.e_shift;
            erow_i = erow_i >= a.e_vocab ? erow_i - a.e_vocab : erow_i;
            const char* erow = (const char*)a.e_w + (size_t)(erow_i >> 4) * a.e_tk * kTileBytes + (erow_i & 15) * 16;
            const float* pe = a.e_pe ? a.e_pe + (size_t)base * K : nullptr;
            auto gather = [&](int k4) -> float4 {
                const int k = k4 * 4;
                float4 v;
                if (DT) {  // 8 inputs per lane chunk: tile k / 32, chunk (k % 32) / 8, half k % 8
                    const uint2 raw = *(const uint2*)(erow + (size_t)(k >> 5) * kTileBytes + ((k & 31) >> 3) * 256 + (k & 7) * 2);
                    v = make_float4(bf2f(raw.x & 0xFFFFu), bf2f(raw.x >> 16), bf2f(raw.y & 0xFFFFu), bf2f(raw.y >> 16));
                } else {   // 4 inputs per lane chunk: tile k / 16, chunk (k % 16) / 4
                    v = *(const float4*)(erow + (size_t)(k >> 4) * kTileBytes + ((k & 15) >> 2) * 256);
                }
                return v;
            };
            float ssj = 0.f;
            for (int kb = tid; kb < n4; kb += 2 * nthr) {
                const int ca = min(kb, n4 - 1), cb = min(kb + nthr, n4 - 1);
                const float4 ea = gather(ca), eb = gather(cb);
                float4 pa = make_float4(0.f, 0.f, 0.f, 0.f), pb = pa;
                if (pe) { pa = *(const float4*)(pe + ca * 4); pb = *(const float4*)(pe + cb * 4); }
                const float4 ga = ldg(ca), gb = ldg(cb);
                XV va, vb;
                // (the embedding kernel's arithmetic: one fused multiply-add of value, scale and position term)
                const float sc = a.e_scale;
                va.p[0] = make_float4(__builtin_fmaf(ea.x, sc, pa.x), __builtin_fmaf(ea.y, sc, pa.y), __builtin_fmaf(ea.z, sc, pa.z), __builtin_fmaf(ea.w, sc, pa.w));
                vb.p[0] = make_float4(__builtin_fmaf(eb.x, sc, pb.x), __builtin_fmaf(eb.y, sc, pb.y), __builtin_fmaf(eb.z, sc, pb.z), __builtin_fmaf(eb.w, sc, pb.w));
                const float sa = put(0, ca, va, ga), sb = put(0, cb, vb, gb);
                ssj += sa + (kb + nthr < n4 ? sb : 0.f);
            }
            if (norm) {
                const float tot = wave_sum(ssj);
                if (lane == 0) ssq[wave * 32] += tot;
            }
        } else if constexpr (PRE) {
            // both planes are copied as they are: pieces of 16 bytes (8 inputs), rows laid end to end and dealt to all
            // threads; indices past the end are clamped (same value to the same place), so no load is conditional
            const int n8 = kc_len >> 3;
            const int total = T * n8;
            const unsigned magic = 0xFFFFFFFFu / (unsigned)n8 + 1u;
            auto round = [&](auto np, int eb, auto&& hk) {
                constexpr int P = decltype(np)::value;
                u32x4 vh[P], vl[P];
                int tt[P], kk[P];
#pragma unroll
                for (int u = 0; u < P; ++u) {
                    const int e = min(eb + u * nthr, total - 1);
                    tt[u] = (int)__umulhi((unsigned)e, magic);
                    kk[u] = e - tt[u] * n8;
                    const size_t off = (size_t)tt[u] * a.ldx + k0 + kk[u] * 8;
                    vh[u] = *(const u32x4*)(a.xb_hi + off);
                    vl[u] = *(const u32x4*)(a.xb_lo + off);
                }
                hk(true);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < P; ++u) {
                    *(u32x4*)(xs_hi + tt[u] * rstride + kk[u] * 16) = vh[u];
                    *(u32x4*)(xs_lo + tt[u] * rstride + kk[u] * 16) = vl[u];
                }
            };
            if (total <= nthr) {
                round(std::integral_constant<int, 1>{}, tid, hook);
            } else if (total <= 2 * nthr) {
                round(std::integral_constant<int, 2>{}, tid, hook);
            } else if (total <= 4 * nthr) {
                round(std::integral_constant<int, 4>{}, tid, hook);
            } else {
                hook(false);
                for (int eb = tid; eb < total; eb += nthr * 4) round(std::integral_constant<int, 4>{}, eb, noop);
            }
        } else if (MG > 0) {
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
                        w[sp] = (m[sp] == -INFINITY) ? 0.f : fexp(m[sp] - M);
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
                    XV rv;
                    rv.p[0] = r;
                    put(tt[u], kk[u], rv, r);
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
                XV v[P];
                float4 g[P];
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
                    const XV va = ldx(t, ca);
                    const float4 ga = ldg(ca);
                    hk(true);
                    __builtin_amdgcn_sched_barrier(0);  // (as above)
                    const float sa = put(t, ca, va, ga);
                    ssj += (act && start < n4) ? sa : 0.f;
                } else if (n4 <= 2 * step) {  // short rows: at most two elements per thread
                    const int ka = start, kb2 = start + step;
                    const int ca = min(ka, n4 - 1), cb = min(kb2, n4 - 1);
                    const XV va = ldx(t, ca), vb = ldx(t, cb);
                    const float4 ga = ldg(ca), gb = ldg(cb);
                    hk(true);
                    __builtin_amdgcn_sched_barrier(0);  // (as above)
                    // unconditional conversions and writes (duplicates carry the same value and count as zero)
                    const float sa = put(t, ca, va, ga), sb = put(t, cb, vb, gb);
                    ssj += (act && ka < n4 ? sa : 0.f) + (act && kb2 < n4 ? sb : 0.f);
                } else if constexpr (PS == 0) {  // (a reader of partial results is launched with at most two pieces per thread)
                    auto rnd = [&](int kb, auto&& hk2) {
                        XV v[8];
                        float4 g[8];
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
            late();
        });
        if (TWO && !second_out) request(B1, wkid + S, nkt0);
        if constexpr (PRE && norm) ssq_request();
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
    } else if (TCAP == 0 && TWO && !ONE) {  // (the few-rows, single-row and single-buffer kernels are launched on single-chunk inputs only)
        request(B0, wkid, nkt0);
        late();
        if constexpr (PRE && norm) ssq_request();
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
    if constexpr (PRE && norm) ssq_reduce();
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
        // Both reductions run over a number of waves known only at run time (at most 8).  Written as loops of that length
        // they become a chain of LDS reads each waited for on its own; unrolled to 8 with a clamped index and the
        // surplus terms dropped (x + 0 is x: the sums and their order are unchanged) the reads go out together.
        if (norm) {
            const float inv_k = __builtin_amdgcn_rcpf((float)K);
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                if (nt < NT) {
                    const int t = min(nt * 16 + tok_l, T - 1);
                    float sum = 0.f;
#pragma unroll
                    for (int w = 0; w < 8; ++w) {
                        const float v = ssq[min(w, NWV - 1) * 32 + t];
                        sum += (w < NWV) ? v : 0.f;
                    }
                    rsc[nt] = __builtin_amdgcn_rsqf(sum * inv_k + a.eps);  // (the argument is at least eps: no denormal handling)
                }
            }
        }
        if (WK > 1) {
            if constexpr (ONE || TCAP > 0) {
                // (single-row launches, four or eight input slices as a rule; with several rows there are fewer slices and
                // more tiles per wave, and the surplus reads cost more than the chain: measured)
#pragma unroll
                for (int w2 = 1; w2 < 8; ++w2) {
                    const int wc = wave + min(w2, WK - 1);
#pragma unroll
                    for (int r = 0; r < RW; ++r) {
                        const f32x4 v = red[(wc * nacc + r * NT) * 64 + lane];
                        if (w2 < WK) acc[r][0] += v;
                    }
                }
            } else {
                for (int w2 = 1; w2 < WK; ++w2)
#pragma unroll
                    for (int r = 0; r < RW; ++r)
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            if (j < NT) acc[r][j] += red[((wave + w2) * nacc + r * NT + j) * 64 + lane];
            }
        }
    }
    // ---- epilogue: lane holds features f = tile*16 + kq*4 + v for row t = nt*16 + tok_l ----
    Stat st[2] = {stat_neutral(), stat_neutral()};
    float nx_ss[2] = {0.f, 0.f};
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
                if constexpr (NX) put_planes(a, t, f0, o);
                else st_act4(a.out + (size_t)t * a.ldo + f0, make_float4(o[0], o[1], o[2], o[3]));
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
                case EPI_PART:
                    st_act4(a.out + (size_t)t * a.ldo + n0, make_float4(v4[0], v4[1], v4[2], v4[3]));
                    break;
                case EPI_RESID: {
                    const float4 o = old[rwi][nt];
                    const float xn[4] = {o.x + v4[0], o.y + v4[1], o.z + v4[2], o.w + v4[3]};
                    st_act4(a.out + (size_t)t * a.ldo + n0, make_float4(xn[0], xn[1], xn[2], xn[3]));
                    if constexpr (NX) {  // the next projection reads x * gain as bf16 planes and the sum of x^2 beside them
                        const float4 gn = *(const float4*)(a.nx_gain + n0);
                        const float w[4] = {xn[0] * gn.x, xn[1] * gn.y, xn[2] * gn.z, xn[3] * gn.w};
                        put_planes(a, t, n0, w);
                        nx_ss[nt] += xn[0] * xn[0] + xn[1] * xn[1] + xn[2] * xn[2] + xn[3] * xn[3];
                    }
                } break;
                case EPI_ACT: {
                    const float o[4] = {fmaxf(v4[0], 0.f), fmaxf(v4[1], 0.f), fmaxf(v4[2], 0.f), fmaxf(v4[3], 0.f)};
                    if constexpr (NX) put_planes(a, t, n0, o);
                    else st_act4(a.out + (size_t)t * a.ldo + n0, make_float4(o[0], o[1], o[2], o[3]));
                } break;
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
    if constexpr (NX && EPI == EPI_RESID) {
        // one partial per owner wave and row: the four lane groups of a row are added in a fixed order
        if (owner) {
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                if (nt >= NT) continue;
                float ss = nx_ss[nt];
                ss = quad_rows_sum(ss);
                const int t = nt * 16 + tok_l;
                if (kq == 0 && t < T) st_act(a.nx_ssq + (size_t)(vblock * WR + wrid) * kMaxRows + t, ss);
            }
        }
    }
    if (epi == EPI_LMHEAD) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            st[nt] = stat_quad_rows(st[nt]);
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

}  // namespace bild
