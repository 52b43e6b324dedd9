// Dense-tile GEMM for passes over MANY rows (more than 512): long sources and the prompt prefill of a
// decoder-only model (the step right in front of the decoding loop: Section 3.2 conditions both models on the
// input x; Section 4.1 measures latency end to end per example, so this step is inside the measured quantity).
//
//   y[M][N] = f(x[M][K]) W^T  with the same fused prologue (RMSNorm) and epilogues (store, residual add, activation /
//   gating, Q/K/V split with RoPE and cache append) as the skinny decode GEMM.
//
// Unlike the decode GEMM, this one is a real dense contraction: with hundreds of rows per weight tile the matrix
// cores, not the weight stream, are the resource to keep busy.  A workgroup of 4 waves owns a tile of 64 rows x
// (4 waves x RW feature tiles x 16) features and walks K in chunks of 128 inputs:
//   - the chunk of activations is normalised, scaled by the gain, split into high and low bf16 parts (two MFMAs per
//     weight tile keep fp32-grade accuracy, as in the decode GEMM) and written ONCE to LDS as the MFMA B operand,
//     64 rows deep, so every weight tile a wave loads feeds 4 row tiles x 2 MFMAs;
//   - weights arrive in HBM already in A-operand register order (bild::TMat), so a wave loads its 1 KiB tiles
//     straight into operand registers - no LDS round trip for A.  The tiles of the next chunk are requested while
//     the current one is multiplied;
//   - the LDS footprint (34 KiB) and register count let two workgroups share a compute unit: one converts while
//     the other multiplies, and the loads of both are in flight together (a compute unit's load rate is set
//     by the bytes it has in flight).
// Row blocks of one feature group re-read its weight tiles from L2 / the memory-side cache; blockIdx.x walks the
// feature groups fastest, so the row blocks that are resident together share them.
#include "kernel_common.h"

namespace bild {

__host__ __device__ constexpr int dense_row_stride(int dt) { return dt ? (dense_kc(1) + 8) * 2 : (dense_kc(0) + 4) * 4; }  // LDS bytes per row

size_t dense_lds_bytes(int dt) { return (size_t)kDenseRows * dense_row_stride(dt) * (dt ? 2 : 1) + kDenseRows * sizeof(float); }

// Sums of the two 32-lane halves of a wavefront (DPP path): lanes 0..31 -> lo, lanes 32..63 -> hi.
__device__ __forceinline__ void half_wave_sums(float v, float& lo, float& hi) {
    v += dpp_f<0xB1, 0xF>(0.f, v);
    v += dpp_f<0x4E, 0xF>(0.f, v);
    v += dpp_f<0x141, 0xF>(0.f, v);
    v += dpp_f<0x140, 0xF>(0.f, v);
    v += dpp_f<0x142, 0xA>(0.f, v);  // row_bcast15: lane 31 holds lanes 0..31, lane 63 holds lanes 32..63
    lo = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 31));
    hi = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// GATED: feature tiles 2j / 2j+1 hold the gate and the linear branch of output feature block j (RW is even).
template <int DT, int RW, int EPI, int ROPE, bool GATED>
__global__ __launch_bounds__(256, 2) void gemm_dense_kernel(const GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int KT = DT ? 32 : 16, KC = dense_kc(DT), NKT = KC / KT, NTR = kDenseRows / 16;
    constexpr int RS = dense_row_stride(DT);
    constexpr bool norm = EPI != EPI_RESID;  // residual-adding projections read un-normalised input (as in the decode GEMM)
    constexpr int PPR = KC / 4;              // float4 pieces per row and chunk (32)
    constexpr int RPI = 64 / PPR;            // rows a wave stages per round (2: one per half wave)
    constexpr int ROUNDS = kDenseRows / (kDenseWaves * RPI);
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r0 = (int)blockIdx.y * kDenseRows;
    const int T = min(kDenseRows, a.T - r0);  // rows of this block that exist
    const float* x = a.x + (size_t)r0 * a.ldx;
    const int K = a.W.k;
    const int tile0 = ((int)blockIdx.x * kDenseWaves + wave) * RW;
    char* xs_hi = smem;
    char* xs_lo = smem + kDenseRows * RS;  // bf16 only
    float* ssq = (float*)(smem + kDenseRows * RS * (DT ? 2 : 1));
    const int tok_l = lane & 15, kq = lane >> 4;
    bool valid[RW];
    const char* wbase[RW];
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        valid[r] = tile0 + r < a.W.tn;
        wbase[r] = (const char*)a.W.w + ((size_t)min(tile0 + r, a.W.tn - 1) * a.W.tk) * kTileBytes;
    }
    const unsigned lane16 = (unsigned)lane * 16u;
    f32x4 acc[RW][NTR];
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int j = 0; j < NTR; ++j) acc[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Staging: lane (k4 = lane % PPR, rsub = lane / PPR) of wave w converts piece k4 of rows w*RPI + rsub + u*4*RPI,
    // u = 0..ROUNDS-1 - the same rows in every chunk, so the sums of squares stay in registers until the end.
    // The pieces of the NEXT chunk are requested before the current one is multiplied: their trip from memory
    // (they were written by the previous kernel, on other XCDs) overlaps with the MFMAs.
    const int k4 = lane % PPR, rsub = lane / PPR;
    float4 xr[ROUNDS], g = make_float4(1.f, 1.f, 1.f, 1.f);
    float ssr[ROUNDS];
#pragma unroll
    for (int u = 0; u < ROUNDS; ++u) ssr[u] = 0.f;
    auto request_x = [&](int k0) {
        const int kc_len = min(KC, K - k0);
        const int k4c = k4 * 4 < kc_len ? k4 : 0;  // a piece past a short last chunk re-reads piece 0 (never used)
        if (norm) g = *(const float4*)(a.gain + k0 + k4c * 4);
#pragma unroll
        for (int u = 0; u < ROUNDS; ++u) {
            const int row = wave * RPI + rsub + u * kDenseWaves * RPI;
            xr[u] = *(const float4*)(x + (size_t)min(row, T - 1) * a.ldx + k0 + k4c * 4);  // rows past the end repeat the last one
        }
    };
    // This wave's weight tiles of a chunk (a tile index past the end reads a clamped, valid address and is never
    // multiplied), one register set: input tile u of the NEXT chunk is requested into the registers of tile u right
    // behind the products that read them, a whole chunk of products before it is needed.
    uint4 W[RW][NKT];
    auto request_w = [&](int k0, int u) {
        const int ktc = min(k0 / KT + u, a.W.tk - 1);
#pragma unroll
        for (int r = 0; r < RW; ++r) W[r][u] = *(const uint4*)(wbase[r] + (size_t)ktc * kTileBytes + lane16);
    };
    request_x(0);
#pragma unroll
    for (int u = 0; u < NKT; ++u) request_w(0, u);

    for (int k0 = 0; k0 < K; k0 += KC) {
        const int kc_len = min(KC, K - k0), nkt = kc_len / KT;
        if (k0) __syncthreads();  // the previous chunk's readers are done
        // ---- x[:, k0 : k0 + kc_len] (times the norm gain) into LDS as the B operand ----
        {
            const bool kin = k4 * 4 < kc_len;
#pragma unroll
            for (int u = 0; u < ROUNDS; ++u) {
                const int row = wave * RPI + rsub + u * kDenseWaves * RPI;
                float4 w = xr[u];
                if (kin) {
                    if (norm) {
                        ssr[u] += w.x * w.x + w.y * w.y + w.z * w.z + w.w * w.w;
                        w.x *= g.x; w.y *= g.y; w.z *= g.z; w.w *= g.w;
                    }
                    if (DT) {
                        uint32_t h01, l01, h23, l23;
                        split_bf16x2(w.x, w.y, h01, l01);
                        split_bf16x2(w.z, w.w, h23, l23);
                        *(uint2*)(xs_hi + row * RS + k4 * 8) = make_uint2(h01, h23);
                        *(uint2*)(xs_lo + row * RS + k4 * 8) = make_uint2(l01, l23);
                    } else {
                        *(float4*)(xs_hi + row * RS + k4 * 16) = w;
                    }
                }
            }
        }
        const bool more = k0 + KC < K;
        if (more) request_x(k0 + KC);
        __syncthreads();
        // ---- multiply: every weight tile against the 4 row tiles of the chunk ----
#pragma unroll
        for (int u = 0; u < NKT; ++u) {
            if (u < nkt) {  // (wave-uniform)
#pragma unroll
                for (int j = 0; j < NTR; ++j) {
                    const int t = j * 16 + tok_l;
                    if (DT) {
                        const bf16x8 Bh = __builtin_bit_cast(bf16x8, *(const uint4*)(xs_hi + t * RS + (u * 32 + kq * 8) * 2));
                        const bf16x8 Bl = __builtin_bit_cast(bf16x8, *(const uint4*)(xs_lo + t * RS + (u * 32 + kq * 8) * 2));
#pragma unroll
                        for (int r = 0; r < RW; ++r)
                            acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, W[r][u]), Bh, acc[r][j], 0, 0, 0);
#pragma unroll
                        for (int r = 0; r < RW; ++r)
                            acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, W[r][u]), Bl, acc[r][j], 0, 0, 0);
                    } else {
                        const float4 b = *(const float4*)(xs_hi + t * RS + (u * 16 + kq * 4) * 4);
                        const float bb[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
                        for (int r = 0; r < RW; ++r) {
                            const float aa[4] = {__uint_as_float(W[r][u].x), __uint_as_float(W[r][u].y),
                                                 __uint_as_float(W[r][u].z), __uint_as_float(W[r][u].w)};
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(aa[q], bb[q], acc[r][j], 0, 0, 0);
                        }
                    }
                }
            }
            if (more) request_w(k0 + KC, u);
        }
    }
    // ---- sums of squares of the rows: each row was staged by the lanes of one wave (half a wave for fp32) ----
    if (norm) {
#pragma unroll
        for (int u = 0; u < ROUNDS; ++u) {
            const int row = wave * RPI + u * kDenseWaves * RPI;
            if (RPI == 1) {
                const float tot = wave_sum(ssr[u]);
                if (lane == 0) ssq[row] = tot;
            } else {
                float lo, hi;
                half_wave_sums(ssr[u], lo, hi);
                if (lane == 0) { ssq[row] = lo; ssq[row + 1] = hi; }
            }
        }
        __syncthreads();
    }

    // ---- epilogue: lane holds features f = tile*16 + kq*4 + v of row t = j*16 + tok_l ----
    const int pos0 = (a.pos_ptr ? *a.pos_ptr : 0) + a.pos_add + r0;
    float* out = a.out ? a.out + (size_t)r0 * a.ldo : nullptr;
    float* q_out = a.q_out ? a.q_out + (size_t)r0 * a.i_dim : nullptr;
#pragma unroll
    for (int j = 0; j < NTR; ++j) {
        const int t = j * 16 + tok_l;
        if (t >= T) continue;
        const float rs = norm ? rsqrtf(ssq[t] / (float)K + a.eps) : 1.f;
        if (GATED) {
#pragma unroll
            for (int p = 0; p < RW / 2; ++p) {
                if (!valid[2 * p + 1]) continue;
                const int f0 = ((tile0 >> 1) + p) * 16 + kq * 4;
                float o[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float gt = acc[2 * p][j][v] * rs, up = acc[2 * p + 1][j][v] * rs;
                    o[v] = (a.act == BILD_ACT_GATED_GELU ? gelu_tanh_f(gt) : silu_f(gt)) * up;
                }
                *(float4*)(out + (size_t)t * a.ldo + f0) = make_float4(o[0], o[1], o[2], o[3]);
            }
            continue;
        }
#pragma unroll
        for (int r = 0; r < RW; ++r) {
            if (!valid[r]) continue;
            const int n0 = (tile0 + r) * 16 + kq * 4;
            float v4[4] = {acc[r][j][0] * rs, acc[r][j][1] * rs, acc[r][j][2] * rs, acc[r][j][3] * rs};
            if (EPI == EPI_STORE) {
                *(float4*)(out + (size_t)t * a.ldo + n0) = make_float4(v4[0], v4[1], v4[2], v4[3]);
            } else if (EPI == EPI_RESID) {
                float4* p = (float4*)(out + (size_t)t * a.ldo + n0);
                const float4 o = *p;
                *p = make_float4(o.x + v4[0], o.y + v4[1], o.z + v4[2], o.w + v4[3]);
            } else if (EPI == EPI_ACT) {
                *(float4*)(out + (size_t)t * a.ldo + n0) =
                    make_float4(fmaxf(v4[0], 0.f), fmaxf(v4[1], 0.f), fmaxf(v4[2], 0.f), fmaxf(v4[3], 0.f));
            } else if (EPI == EPI_QKV) {
                const int pos = pos0 + t;
                const int seg = n0 < a.q_dim ? 0 : (n0 < a.q_dim + a.i_dim ? 1 : 2);
                const int nn = n0 - (seg == 0 ? 0 : (seg == 1 ? a.q_dim : a.q_dim + a.i_dim));
                if (ROPE && seg < 2) {  // pairs (2i, 2i+1) of a head rotate by position * base^(-2i/d_head)
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
                    *(float4*)(q_out + (size_t)t * a.i_dim + nn) = make_float4(v4[0], v4[1], v4[2], v4[3]);
                } else if (seg == 1) {  // K: [position][I]
                    const size_t e = (size_t)pos * a.i_dim + nn;
                    if (DT)
                        *(uint2*)((uint16_t*)a.k_cache + e) = make_uint2(pack_bf16x2(v4[0], v4[1]), pack_bf16x2(v4[2], v4[3]));
                    else
                        *(float4*)((float*)a.k_cache + e) = make_float4(v4[0], v4[1], v4[2], v4[3]);
                } else {  // V: transposed, [I][vcap] with the position contiguous
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const size_t e = (size_t)(nn + v) * a.vcap + pos;
                        if (DT)
                            ((uint16_t*)a.v_cache)[e] = (uint16_t)f2bf(v4[v]);
                        else
                            ((float*)a.v_cache)[e] = v4[v];
                    }
                }
            }
        }
    }
}

size_t dense_num_feature_groups(const GemmArgs& a) {
    const int per = kDenseWaves * kDenseRW;
    return (size_t)(a.W.tn + per - 1) / per;
}

hipError_t launch_gemm_dense(const GemmArgs& a, int dtype, hipStream_t st) {
    static hipError_t attr = [] {
        const void* fns[] = {
#define BILD_DENSE(DTV)                                                                                             \
    (const void*)gemm_dense_kernel<DTV, kDenseRW, EPI_STORE, 0, false>, (const void*)gemm_dense_kernel<DTV, kDenseRW, EPI_RESID, 0, false>, \
    (const void*)gemm_dense_kernel<DTV, kDenseRW, EPI_QKV, 0, false>, (const void*)gemm_dense_kernel<DTV, kDenseRW, EPI_QKV, 1, false>,     \
    (const void*)gemm_dense_kernel<DTV, kDenseRW, EPI_ACT, 0, false>, (const void*)gemm_dense_kernel<DTV, kDenseRW, EPI_ACT, 0, true>
            BILD_DENSE(0), BILD_DENSE(1)};
#undef BILD_DENSE
        for (const void* f : fns) {
            hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }();
    if (attr != hipSuccess) return attr;
    if (a.T < 1 || a.W.k < 1 || a.epi == EPI_LMHEAD || a.mg_splits > 1) return hipErrorInvalidValue;
    if ((a.gain != nullptr) != (a.epi != EPI_RESID)) return hipErrorInvalidValue;  // the norm is fixed by the epilogue
    const bool gated = a.epi == EPI_ACT && a.act != BILD_ACT_RELU;
    const dim3 grid((unsigned)dense_num_feature_groups(a), (unsigned)((a.T + kDenseRows - 1) / kDenseRows)), block(64 * kDenseWaves);
    const size_t smem = dense_lds_bytes(dtype);
#define BILD_DL(DTV)                                                                                                        \
    switch (a.epi) {                                                                                                        \
        case EPI_STORE: hipLaunchKernelGGL((gemm_dense_kernel<DTV, kDenseRW, EPI_STORE, 0, false>), grid, block, smem, st, a); break; \
        case EPI_RESID: hipLaunchKernelGGL((gemm_dense_kernel<DTV, kDenseRW, EPI_RESID, 0, false>), grid, block, smem, st, a); break; \
        case EPI_QKV:                                                                                                       \
            if (a.rope) hipLaunchKernelGGL((gemm_dense_kernel<DTV, kDenseRW, EPI_QKV, 1, false>), grid, block, smem, st, a);  \
            else hipLaunchKernelGGL((gemm_dense_kernel<DTV, kDenseRW, EPI_QKV, 0, false>), grid, block, smem, st, a);         \
            break;                                                                                                          \
        case EPI_ACT:                                                                                                       \
            if (gated) hipLaunchKernelGGL((gemm_dense_kernel<DTV, kDenseRW, EPI_ACT, 0, true>), grid, block, smem, st, a);    \
            else hipLaunchKernelGGL((gemm_dense_kernel<DTV, kDenseRW, EPI_ACT, 0, false>), grid, block, smem, st, a);         \
            break;                                                                                                          \
        default: return hipErrorInvalidValue;                                                                               \
    }
    if (dtype) { BILD_DL(1) } else { BILD_DL(0) }
#undef BILD_DL
    return hipGetLastError();
}

}  // namespace bild
