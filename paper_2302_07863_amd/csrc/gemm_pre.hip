// Launch wrappers of the skinny GEMM for passes whose activations travel between projections as bf16 planes
// (bf16 models, up to 32 rows).  The kernel that produces an activation splits every value once into a high and a
// low bf16 part (with the gain of the consumer's RMSNorm applied) and leaves the sums of squares beside them; the
// consuming workgroups then stage their operand with plain 16-byte copies instead of each converting all rows
// again - in a review of n drafts that conversion, repeated in every workgroup of a projection, was the larger
// part of what the pass cost beyond a single-row step (Section 3.2: n rows, one weight load).
#include "gemm_body.h"

namespace bild {

// Input in planes; residual and activation epilogues hand their output on in planes as well.
template <int RW, int EPI, int ROPE, int NT, bool SHORT = false>
__global__ __launch_bounds__(512) void gemm_pre_kernel(BILD_GEMM_HOT_PARAMS, const GemmArgs a0) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const GemmArgs a = gemm_hot<HOT_PRE, 1>(a0, BILD_GEMM_HOT_NAMES);
    gemm_body<1, RW, EPI, ROPE, NT, gemm_batch(RW, false, NT), 0, false, !SHORT, 0, true,
              EPI == EPI_RESID || EPI == EPI_ACT>(a, (int)blockIdx.x, smem);
}

// Output projection whose input is still in key-split attention partials (fp32, merged while staging); output in planes.
template <int SPLITS, bool SHORT = false>
__global__ __launch_bounds__(512) void gemm_merge_nx_kernel(BILD_GEMM_HOT_PARAMS, const GemmArgs a0) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const GemmArgs a = gemm_hot<HOT_MG, 1>(a0, BILD_GEMM_HOT_NAMES);
    gemm_body<1, 1, EPI_RESID, 0, 1, gemm_batch(1, false), SPLITS, false, !SHORT, 0, false, true>(a, (int)blockIdx.x, smem);
}

hipError_t gemm_pre_init() {
    static hipError_t done = [] {
#define BILD_P1(NTV) \
    (const void*)gemm_pre_kernel<1, EPI_STORE, 0, NTV>, (const void*)gemm_pre_kernel<1, EPI_RESID, 0, NTV>, \
    (const void*)gemm_pre_kernel<1, EPI_QKV, 0, NTV>, (const void*)gemm_pre_kernel<1, EPI_QKV, 1, NTV>, \
    (const void*)gemm_pre_kernel<1, EPI_ACT, 0, NTV>, (const void*)gemm_pre_kernel<2, EPI_ACT, 0, NTV>, \
    (const void*)gemm_pre_kernel<1, EPI_LMHEAD, 0, NTV>
        const void* fns[] = {BILD_P1(1), BILD_P1(2),
                             (const void*)gemm_pre_kernel<1, EPI_STORE, 0, 1, true>, (const void*)gemm_pre_kernel<1, EPI_RESID, 0, 1, true>,
                             (const void*)gemm_pre_kernel<1, EPI_QKV, 0, 1, true>, (const void*)gemm_pre_kernel<1, EPI_QKV, 1, 1, true>,
                             (const void*)gemm_pre_kernel<1, EPI_ACT, 0, 1, true>, (const void*)gemm_pre_kernel<1, EPI_LMHEAD, 0, 1, true>,
                             (const void*)gemm_pre_kernel<4, EPI_LMHEAD, 0, 1>,
                             (const void*)gemm_merge_nx_kernel<2>, (const void*)gemm_merge_nx_kernel<4>, (const void*)gemm_merge_nx_kernel<8>,
                             (const void*)gemm_merge_nx_kernel<2, true>, (const void*)gemm_merge_nx_kernel<4, true>,
                             (const void*)gemm_merge_nx_kernel<8, true>};
#undef BILD_P1
        for (const void* f : fns) {
            hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }();
    return done;
}

// `a` has its launch shape (gemm_pick_shape) and either input planes (xb_hi) or key-split partials with output planes.
hipError_t launch_gemm_pre(const GemmArgs& a, hipStream_t st) {
    if (hipError_t e = gemm_pre_init(); e != hipSuccess) return e;
    if (a.T < 1 || a.T > kMaxRows) return hipErrorInvalidValue;
    const bool hands_on = a.epi == EPI_RESID || a.epi == EPI_ACT;
    if (hands_on != (a.nx_hi != nullptr) || (hands_on && (!a.nx_lo || a.nx_ld < a.W.n / a.rw))) return hipErrorInvalidValue;
    if (a.epi == EPI_RESID && (!a.nx_gain || !a.nx_ssq)) return hipErrorInvalidValue;
    const size_t smem = gemm_lds_bytes(a, 1);
    const dim3 grid((unsigned)gemm_num_blocks(a)), block(64 * a.nwv);
    const bool one_chunk = a.W.k <= a.kc;
    const int per_wave = (a.W.tk + a.wk - 1) / a.wk;
    const bool sh = one_chunk && per_wave <= gemm_batch(1, false);  // one batch of tiles per wave at most: no second buffer
    if (!a.xb_hi) {
        const int sp = a.mg_splits, npairs = a.T * a.mg_heads;
        if ((sp != 2 && sp != 4 && sp != 8) || a.T > 16 || a.epi != EPI_RESID || a.rw != 1 || a.mg_heads < 1 ||
            npairs > 64 * a.nwv || (size_t)npairs * sp * 4 > (size_t)gemm_red_bytes(a.nwv, 1))
            return hipErrorInvalidValue;
#define BILD_MG(SH)                                                                              \
    do {                                                                                          \
        if (sp == 2) hipLaunchKernelGGL((gemm_merge_nx_kernel<2, SH>), grid, block, smem, st, BILD_GEMM_HOT_MG(a), a); \
        else if (sp == 4) hipLaunchKernelGGL((gemm_merge_nx_kernel<4, SH>), grid, block, smem, st, BILD_GEMM_HOT_MG(a), a); \
        else hipLaunchKernelGGL((gemm_merge_nx_kernel<8, SH>), grid, block, smem, st, BILD_GEMM_HOT_MG(a), a);         \
    } while (0)
        if (sh) BILD_MG(true); else BILD_MG(false);
#undef BILD_MG
        return hipGetLastError();
    }
    if (!a.xb_lo || (a.W.k & 7) || (a.ldx & 7)) return hipErrorInvalidValue;
    // normed input: the producer's partial sums of squares, at most 256 of them, rows dealt to the waves (see ssq_request)
    if ((a.epi != EPI_RESID) && (!a.ssq_part || a.ssq_parts < 1 || a.ssq_parts > kMaxSsqParts || a.T > (a.T > 16 ? 8 : 4) * a.nwv))
        return hipErrorInvalidValue;
#define BILD_L(RWV, EPIV, ROPEV)                                                                      \
    do {                                                                                               \
        if (a.T > 16) hipLaunchKernelGGL((gemm_pre_kernel<RWV, EPIV, ROPEV, 2>), grid, block, smem, st, BILD_GEMM_HOT_PRE(a), a); \
        else if (RWV == 1 && sh) hipLaunchKernelGGL((gemm_pre_kernel<1, EPIV, ROPEV, 1, true>), grid, block, smem, st, BILD_GEMM_HOT_PRE(a), a); \
        else hipLaunchKernelGGL((gemm_pre_kernel<RWV, EPIV, ROPEV, 1>), grid, block, smem, st, BILD_GEMM_HOT_PRE(a), a);    \
    } while (0)
    switch (a.epi) {
        case EPI_STORE: BILD_L(1, EPI_STORE, 0); break;
        case EPI_RESID: BILD_L(1, EPI_RESID, 0); break;
        case EPI_QKV:
            if (a.rope) BILD_L(1, EPI_QKV, 1); else BILD_L(1, EPI_QKV, 0);
            break;
        case EPI_ACT:
            if (a.rw == 2) BILD_L(2, EPI_ACT, 0); else BILD_L(1, EPI_ACT, 0);
            break;
        case EPI_LMHEAD:
            if (a.rw == 4 && a.T <= 16) hipLaunchKernelGGL((gemm_pre_kernel<4, EPI_LMHEAD, 0, 1>), grid, block, smem, st, BILD_GEMM_HOT_PRE(a), a);
            else if (a.rw != 1) return hipErrorInvalidValue;
            else BILD_L(1, EPI_LMHEAD, 0);
            break;
        default: return hipErrorInvalidValue;
    }
#undef BILD_L
    return hipGetLastError();
}

}  // namespace bild
