// HIP kernels of the BiLD decoding path for gfx950 (CDNA4, wave64).
//
//   gemm_kernel      weight-streaming skinny GEMM  y[T][N] = f(x[T][K]) W^T for T <= 32 rows
//                    (T = 1: the small model's autoregressive step; T = n+1: the large
//                    model's non-autoregressive review, Section 3.2), with the RMSNorm of
//                    the input fused in front and the consumer (K/V cache append + RoPE,
//                    activation, residual add, LM-head softmax statistics) fused behind.
//   attn_kernel      KV-cache attention for T query rows of one head.
//   embed_kernel     embedding gather + sinusoidal position.
//   finish_kernel    merges the LM-head partial statistics and applies the fallback /
//                    rollback policy (Sections 3.3, 3.4; Algorithm 1), committing y and
//                    the cache lengths on the device.
//
// The path is bound by HBM bandwidth: every weight byte is read once per pass and the
// arithmetic per byte is tiny.  Weights therefore sit in HBM in the exact register order
// of the matrix-core A operand (see bild::TMat) so that one wavefront load instruction
// moves 1 KiB of contiguous memory straight into MFMA operand registers; activations
// (a few KiB) are staged once per workgroup in LDS as the B operand.  bf16 models keep
// activations at fp32 accuracy by splitting each value into a high and a low bf16 part
// and issuing two MFMAs per weight tile; the matrix cores have an order of magnitude
// more throughput than the stream needs, so this is free.
#include <hip/hip_runtime.h>
#include <math.h>

#include "bild_internal.h"

namespace bild {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t f2bf(float f) {  // fp32 -> bf16 bits, nearest even
    uint32_t u = __float_as_uint(f);
    return (u + (((u >> 16) & 1u) + 0x7FFFu)) >> 16;
}
__device__ __forceinline__ float bf2f(uint32_t h) { return __uint_as_float(h << 16); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// ---- online softmax statistics ------------------------------------------------------
struct Stat {
    float m, s;
    int idx;
};
__device__ __forceinline__ Stat stat_neutral() { return Stat{-INFINITY, 0.f, 0x7FFFFFFF}; }
__device__ __forceinline__ void stat_push(Stat& a, float z, int n) {
    if (z > a.m) {  // strict: equal maxima keep the lower id (ids arrive in increasing order)
        a.s = a.s * expf(a.m - z) + 1.f;
        a.m = z;
        a.idx = n;
    } else {
        a.s += expf(z - a.m);
    }
}
__device__ __forceinline__ Stat stat_merge(const Stat& a, const Stat& b) {
    Stat r;
    r.m = fmaxf(a.m, b.m);
    const float sa = (a.m == -INFINITY) ? 0.f : a.s * expf(a.m - r.m);
    const float sb = (b.m == -INFINITY) ? 0.f : b.s * expf(b.m - r.m);
    r.s = sa + sb;
    r.idx = (a.m > b.m || (a.m == b.m && a.idx < b.idx)) ? a.idx : b.idx;
    return r;
}
__device__ __forceinline__ Stat stat_shfl_xor(const Stat& a, int o) {
    Stat b;
    b.m = __shfl_xor(a.m, o, 64);
    b.s = __shfl_xor(a.s, o, 64);
    b.idx = __shfl_xor(a.idx, o, 64);
    return b;
}

__device__ __forceinline__ float gelu_tanh_f(float u) {
    return 0.5f * u * (1.f + tanhf(0.7978845608028654f * (u + 0.044715f * u * u * u)));
}
__device__ __forceinline__ float silu_f(float u) { return u / (1.f + expf(-u)); }

// =====================================================================================
// Skinny GEMM.  Workgroup = 4 wavefronts.  The waves are arranged as (4/wk) feature
// groups x wk input slices; each wave owns rw feature tiles (16 features each) and
// walks the input tiles of its slice.  LDS layout (dynamic):
//   [0, xs)        staged activations of the current input chunk
//   red            cross-wave partial sums when wk > 1      (4 x 4 x 64 float4)
//   ssq[4][32]     per-wave sums of squares for the RMSNorm
//   rs[32]         per-row 1/rms
//   wstat[4][32]   per-wave softmax partials (LM head)
// =====================================================================================
constexpr int kRedBytes = 4 * 4 * 64 * 16;
constexpr int kTailBytes = kRedBytes + 4 * 32 * 4 + 32 * 4 + 4 * 32 * 16;

__host__ __device__ inline int xs_row_stride(int dt, int kc) { return dt ? (kc + 8) * 2 : (kc + 4) * 4; }
__host__ __device__ inline int xs_bytes(int dt, int kc, int T) { return T * xs_row_stride(dt, kc) * (dt ? 2 : 1); }

template <int DT>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int KT = DT ? 32 : 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int T = a.T, K = a.W.k, KC = a.kc;
    const int WK = a.wk, WR = 4 / WK, RW = a.rw;
    const int wkid = wave % WK, wrid = wave / WK;
    const int tile0 = ((int)blockIdx.x * WR + wrid) * RW;
    const int NT = (T + 15) >> 4;
    const int rstride = xs_row_stride(DT, KC);
    char* xs_hi = smem;
    char* xs_lo = smem + T * rstride;  // bf16 only
    char* tail = smem + xs_bytes(DT, KC, T);
    f32x4* red = (f32x4*)tail;
    float* ssq = (float*)(tail + kRedBytes);
    float* rs = ssq + 128;
    StatPart* wstat = (StatPart*)(rs + 32);

    const bool norm = a.gain != nullptr;
    const bool few = T < 4;  // few rows: all waves share each row, split along k
    const bool valid0 = tile0 < a.W.tn;
    const bool valid1 = (RW == 2) && (tile0 + 1 < a.W.tn);
    const char* wbase0 = (const char*)a.W.w + ((size_t)tile0 * a.W.tk) * kTileBytes + lane * 16;
    const char* wbase1 = wbase0 + (size_t)a.W.tk * kTileBytes;

    if (tid < 128) ssq[tid] = 0.f;

    f32x4 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    float ss[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) ss[j] = 0.f;

    const int tok_l = lane & 15, kq = lane >> 4;

    for (int k0 = 0; k0 < K; k0 += KC) {
        const int kc_len = min(KC, K - k0);
        if (k0) __syncthreads();  // readers of the previous chunk are done
        // ---- stage x[:, k0 : k0+kc_len] (times the norm gain) into LDS ----
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int t = few ? j : wave + 4 * j;
            if (t < T) {
                const float* xr = a.x + (size_t)t * a.ldx + k0;
                const int start = few ? tid : lane, step = few ? 256 : 64;
                for (int k4 = start; k4 < (kc_len >> 2); k4 += step) {
                    float4 v = *(const float4*)(xr + k4 * 4);
                    if (norm) {
                        ss[j] += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
                        const float4 g = *(const float4*)(a.gain + k0 + k4 * 4);
                        v.x *= g.x; v.y *= g.y; v.z *= g.z; v.w *= g.w;
                    }
                    if (DT) {
                        const uint32_t h0 = f2bf(v.x), h1 = f2bf(v.y), h2 = f2bf(v.z), h3 = f2bf(v.w);
                        const uint32_t l0 = f2bf(v.x - bf2f(h0)), l1 = f2bf(v.y - bf2f(h1));
                        const uint32_t l2 = f2bf(v.z - bf2f(h2)), l3 = f2bf(v.w - bf2f(h3));
                        *(uint2*)(xs_hi + t * rstride + k4 * 8) = make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
                        *(uint2*)(xs_lo + t * rstride + k4 * 8) = make_uint2(l0 | (l1 << 16), l2 | (l3 << 16));
                    } else {
                        *(float4*)(xs_hi + t * rstride + k4 * 16) = v;
                    }
                }
            }
        }
        __syncthreads();
        // ---- stream this wave's weight tiles of the chunk ----
        const int kt_base = k0 / KT, nkt = kc_len / KT;
        auto compute = [&](const uint4& A0, const uint4& A1, int ktl) {
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                if (nt < NT) {
                    const int t = nt * 16 + tok_l;
                    if (DT) {
                        uint4 bh = make_uint4(0, 0, 0, 0), bl = make_uint4(0, 0, 0, 0);
                        if (t < T) {
                            bh = *(const uint4*)(xs_hi + t * rstride + (ktl * 32 + kq * 8) * 2);
                            bl = *(const uint4*)(xs_lo + t * rstride + (ktl * 32 + kq * 8) * 2);
                        }
                        const bf16x8 Bh = __builtin_bit_cast(bf16x8, bh), Bl = __builtin_bit_cast(bf16x8, bl);
                        if (valid0) {
                            const bf16x8 A = __builtin_bit_cast(bf16x8, A0);
                            acc[0][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, Bh, acc[0][nt], 0, 0, 0);
                            acc[0][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, Bl, acc[0][nt], 0, 0, 0);
                        }
                        if (valid1) {
                            const bf16x8 A = __builtin_bit_cast(bf16x8, A1);
                            acc[1][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, Bh, acc[1][nt], 0, 0, 0);
                            acc[1][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, Bl, acc[1][nt], 0, 0, 0);
                        }
                    } else {
                        float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
                        if (t < T) b = *(const float4*)(xs_hi + t * rstride + (ktl * 16 + kq * 4) * 4);
                        const float bb[4] = {b.x, b.y, b.z, b.w};
                        if (valid0) {
                            const float aa[4] = {__uint_as_float(A0.x), __uint_as_float(A0.y), __uint_as_float(A0.z),
                                                 __uint_as_float(A0.w)};
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                acc[0][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(aa[j], bb[j], acc[0][nt], 0, 0, 0);
                        }
                        if (valid1) {
                            const float aa[4] = {__uint_as_float(A1.x), __uint_as_float(A1.y), __uint_as_float(A1.z),
                                                 __uint_as_float(A1.w)};
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                acc[1][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(aa[j], bb[j], acc[1][nt], 0, 0, 0);
                        }
                    }
                }
            }
        };
        int kt = wkid;
        constexpr int U = 4;
        for (; kt + (U - 1) * WK < nkt; kt += U * WK) {
            uint4 A0[U], A1[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const size_t off = (size_t)(kt_base + kt + u * WK) * kTileBytes;
                A0[u] = valid0 ? *(const uint4*)(wbase0 + off) : make_uint4(0, 0, 0, 0);
                A1[u] = valid1 ? *(const uint4*)(wbase1 + off) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) compute(A0[u], A1[u], kt + u * WK);
        }
        for (; kt < nkt; kt += WK) {
            const size_t off = (size_t)(kt_base + kt) * kTileBytes;
            const uint4 A0 = valid0 ? *(const uint4*)(wbase0 + off) : make_uint4(0, 0, 0, 0);
            const uint4 A1 = valid1 ? *(const uint4*)(wbase1 + off) : make_uint4(0, 0, 0, 0);
            compute(A0, A1, kt);
        }
    }

    // ---- RMSNorm row scales and cross-wave k reduction ----
    if (norm) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int t = few ? j : wave + 4 * j;
            const float v = wave_sum(ss[j]);
            if (t < T && lane == 0) ssq[wave * 32 + t] = v;
        }
    }
    if (WK > 1 && wkid > 0) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) red[(wave * 4 + i * 2 + j) * 64 + lane] = acc[i][j];
    }
    __syncthreads();
    if (tid < T)
        rs[tid] = norm ? rsqrtf((ssq[tid] + ssq[32 + tid] + ssq[64 + tid] + ssq[96 + tid]) / (float)K + a.eps) : 1.f;
    if (WK > 1 && wkid == 0) {
        for (int w2 = 1; w2 < WK; ++w2)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] += red[((wave + w2) * 4 + i * 2 + j) * 64 + lane];
    }
    __syncthreads();

    // ---- epilogue: lane holds features f = tile*16 + kq*4 + v for row t = nt*16 + tok_l ----
    const bool owner = (wkid == 0);
    const int pos0 = (a.pos_ptr ? *a.pos_ptr : 0) + a.pos_add;
    Stat st[2] = {stat_neutral(), stat_neutral()};
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int t = nt * 16 + tok_l;
        if (nt >= NT || t >= T || !owner) continue;
        const float r = rs[t];
        if (a.epi == EPI_ACT && a.act != BILD_ACT_RELU) {
            if (valid0 && valid1) {  // tile0 even: gate tile, tile0+1: linear branch of the same features
                const int f0 = (tile0 >> 1) * 16 + kq * 4;
                float o[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float g = acc[0][nt][v] * r, u = acc[1][nt][v] * r;
                    o[v] = (a.act == BILD_ACT_GATED_GELU ? gelu_tanh_f(g) : silu_f(g)) * u;
                }
                *(float4*)(a.out + (size_t)t * a.ldo + f0) = make_float4(o[0], o[1], o[2], o[3]);
            }
            continue;
        }
#pragma unroll
        for (int rwi = 0; rwi < 2; ++rwi) {
            if (!(rwi == 0 ? valid0 : valid1)) continue;
            const int n0 = (tile0 + rwi) * 16 + kq * 4;
            float v4[4] = {acc[rwi][nt][0] * r, acc[rwi][nt][1] * r, acc[rwi][nt][2] * r, acc[rwi][nt][3] * r};
            switch (a.epi) {
                case EPI_STORE:
                    *(float4*)(a.out + (size_t)t * a.ldo + n0) = make_float4(v4[0], v4[1], v4[2], v4[3]);
                    break;
                case EPI_RESID: {
                    float4* p = (float4*)(a.out + (size_t)t * a.ldo + n0);
                    float4 o = *p;
                    o.x += v4[0]; o.y += v4[1]; o.z += v4[2]; o.w += v4[3];
                    *p = o;
                } break;
                case EPI_ACT:
                    *(float4*)(a.out + (size_t)t * a.ldo + n0) =
                        make_float4(fmaxf(v4[0], 0.f), fmaxf(v4[1], 0.f), fmaxf(v4[2], 0.f), fmaxf(v4[3], 0.f));
                    break;
                case EPI_QKV: {
                    const int pos = pos0 + t;
                    const int seg = n0 < a.q_dim ? 0 : (n0 < a.q_dim + a.i_dim ? 1 : 2);
                    const int nn = n0 - (seg == 0 ? 0 : (seg == 1 ? a.q_dim : a.q_dim + a.i_dim));
                    if (a.rope && seg < 2) {
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
                        *(float4*)(a.q_out + (size_t)t * a.i_dim + nn) = make_float4(v4[0], v4[1], v4[2], v4[3]);
                    } else {
                        void* cache = seg == 1 ? a.k_cache : a.v_cache;
                        const size_t e = (size_t)pos * a.i_dim + nn;
                        if (DT)
                            *(uint2*)((uint16_t*)cache + e) =
                                make_uint2(f2bf(v4[0]) | (f2bf(v4[1]) << 16), f2bf(v4[2]) | (f2bf(v4[3]) << 16));
                        else
                            *(float4*)((float*)cache + e) = make_float4(v4[0], v4[1], v4[2], v4[3]);
                    }
                } break;
                case EPI_LMHEAD: {
                    const int row = a.row_off + t;
                    const int ti = pos0 + t + 1;
                    const int tgt = (ti < *a.ylen_ptr) ? a.y[ti] : -1;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int n = n0 + v;
                        if (n < a.vocab) {
                            const float z = v4[v] * a.scale;
                            stat_push(st[nt], z, n);
                            if (n == tgt) a.zt[row] = z;
                            if (a.dbg) a.dbg[(size_t)row * a.vocab + n] = z;
                        }
                    }
                } break;
            }
        }
    }
    if (a.epi == EPI_LMHEAD) {
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
            for (int w = 0; w < 4; ++w) {
                const StatPart sp = wstat[w * 32 + tid];
                r = stat_merge(r, Stat{sp.m, sp.s, sp.idx});
            }
            StatPart o;
            o.m = r.m; o.s = r.s; o.idx = r.idx; o.pad = 0;
            a.part[(size_t)blockIdx.x * kMaxRows + a.row_off + tid] = o;
        }
    }
}

void gemm_pick_shape(GemmArgs& a, int dtype) {
    const int kt = dtype ? 32 : 16;
    const bool gated = a.epi == EPI_ACT && a.act != BILD_ACT_RELU;
    a.rw = gated ? 2 : 1;
    int kc = 16384 / a.T - 8;
    kc = (kc / 128) * 128;
    if (kc < 128) kc = 128;
    if (kc > a.W.k) kc = a.W.k;
    a.kc = kc;
    int wk = 1;
    const int tiles_chunk = kc / kt;
    while (wk < 4 && (a.W.tn + (4 / wk) * a.rw - 1) / ((4 / wk) * a.rw) < 512 && tiles_chunk / (wk * 2) >= 2) wk *= 2;
    a.wk = wk;
}

size_t gemm_num_blocks(const GemmArgs& a) {
    const int per = (4 / a.wk) * a.rw;
    return (size_t)(a.W.tn + per - 1) / per;
}

template <int DT>
__global__ void attn_kernel(const AttnArgs a);

// Both big kernels may ask for more than the default 64 KiB of dynamic LDS.
static hipError_t raise_lds_limits() {
    static hipError_t done = [] {
        const int lim = 128 * 1024;
        hipError_t e = hipFuncSetAttribute((const void*)gemm_kernel<0>, hipFuncAttributeMaxDynamicSharedMemorySize, lim);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void*)gemm_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, lim);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void*)attn_kernel<0>, hipFuncAttributeMaxDynamicSharedMemorySize, lim);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void*)attn_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, lim);
        return e;
    }();
    return done;
}

hipError_t launch_gemm(const GemmArgs& a, int dtype, hipStream_t st) {
    if (hipError_t e = raise_lds_limits(); e != hipSuccess) return e;
    const size_t smem = (size_t)xs_bytes(dtype, a.kc, a.T) + kTailBytes;
    const dim3 grid((unsigned)gemm_num_blocks(a));
    if (dtype)
        hipLaunchKernelGGL(gemm_kernel<1>, grid, dim3(256), smem, st, a);
    else
        hipLaunchKernelGGL(gemm_kernel<0>, grid, dim3(256), smem, st, a);
    return hipGetLastError();
}

// =====================================================================================
// Attention over a position-major cache [position][I].  One workgroup per (head, key
// split); all T query rows share each K/V load.  Keys are processed 256 at a time:
// one thread per key computes the T scores, the waves update the running (max, sum)
// of their rows, then threads re-map to (key part, head dim) for the P V product.
// =====================================================================================
template <int DT>
__global__ __launch_bounds__(256) void attn_kernel(const AttnArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int T = a.T, dh = a.d_head, I = a.i_dim;
    const int h = blockIdx.x, sp = blockIdx.y;
    float* q_s = (float*)smem;              // [T][dh]
    float* S = q_s + T * dh;                // [T][256]
    float* m_s = S + T * 256;               // [T]
    float* l_s = m_s + kMaxRows;            // [T]
    float* f_s = l_s + kMaxRows;            // [T]
    float* red = f_s + kMaxRows;            // [nparts][T][dh]

    const int base = a.causal ? (*a.base_ptr + a.base_add) : 0;
    const int nkeys = a.causal ? base + T : (a.nkeys_ptr ? *a.nkeys_ptr : a.nkeys_fixed);
    int per = (nkeys + a.splits - 1) / a.splits;
    per = ((per + 255) / 256) * 256;
    const int k_begin = min(nkeys, sp * per), k_end = min(nkeys, k_begin + per);

    for (int i = tid; i < T * dh; i += 256) q_s[i] = a.q[(size_t)(i / dh) * I + h * dh + (i % dh)] * a.scale;
    if (tid < T) {
        m_s[tid] = -INFINITY;
        l_s[tid] = 0.f;
    }
    const int nparts = 256 / dh;
    const int pd = tid % dh, part = tid / dh;
    float acc[kMaxRows];
#pragma unroll
    for (int t = 0; t < kMaxRows; ++t) acc[t] = 0.f;
    __syncthreads();

    for (int c0 = k_begin; c0 < k_end; c0 += 256) {
        const int key = c0 + tid;
        const bool kvalid = key < k_end;
        // ---- scores of this thread's key against every row ----
        float s[kMaxRows];
#pragma unroll
        for (int t = 0; t < kMaxRows; ++t) s[t] = 0.f;
        if (kvalid) {
            for (int seg = 0; seg < dh; seg += 8) {
                float kf[8];
                if (DT) {
                    const uint4 u = *(const uint4*)((const uint16_t*)a.k + (size_t)key * I + h * dh + seg);
                    kf[0] = bf2f(u.x & 0xFFFF); kf[1] = bf2f(u.x >> 16);
                    kf[2] = bf2f(u.y & 0xFFFF); kf[3] = bf2f(u.y >> 16);
                    kf[4] = bf2f(u.z & 0xFFFF); kf[5] = bf2f(u.z >> 16);
                    kf[6] = bf2f(u.w & 0xFFFF); kf[7] = bf2f(u.w >> 16);
                } else {
                    const float4 u0 = *(const float4*)((const float*)a.k + (size_t)key * I + h * dh + seg);
                    const float4 u1 = *(const float4*)((const float*)a.k + (size_t)key * I + h * dh + seg + 4);
                    kf[0] = u0.x; kf[1] = u0.y; kf[2] = u0.z; kf[3] = u0.w;
                    kf[4] = u1.x; kf[5] = u1.y; kf[6] = u1.z; kf[7] = u1.w;
                }
#pragma unroll
                for (int t = 0; t < kMaxRows; ++t) {
                    if (t < T) {
                        const float4 qa = *(const float4*)(q_s + t * dh + seg);
                        const float4 qb = *(const float4*)(q_s + t * dh + seg + 4);
                        s[t] += qa.x * kf[0] + qa.y * kf[1] + qa.z * kf[2] + qa.w * kf[3] + qb.x * kf[4] + qb.y * kf[5] +
                                qb.z * kf[6] + qb.w * kf[7];
                    }
                }
            }
        }
#pragma unroll
        for (int t = 0; t < kMaxRows; ++t)
            if (t < T) S[t * 256 + tid] = (kvalid && (!a.causal || key <= base + t)) ? s[t] : -INFINITY;
        __syncthreads();
        // ---- running max / sum per row; scores become probabilities relative to the new max ----
        for (int t = wave; t < T; t += 4) {
            float v[4], mx = -INFINITY;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[i] = S[t * 256 + lane + 64 * i];
                mx = fmaxf(mx, v[i]);
            }
            mx = wave_max(mx);
            const float m_old = m_s[t], m_new = fmaxf(m_old, mx);
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float p = (m_new == -INFINITY) ? 0.f : expf(v[i] - m_new);
                S[t * 256 + lane + 64 * i] = p;
                sum += p;
            }
            sum = wave_sum(sum);
            if (lane == 0) {
                const float f = (m_old == -INFINITY) ? 0.f : expf(m_old - m_new);
                f_s[t] = f;
                l_s[t] = l_s[t] * f + sum;
                m_s[t] = m_new;
            }
        }
        __syncthreads();
        // ---- acc[t][pd] += sum over this part's keys of P[t][key] * V[key][pd] ----
        if (part < nparts) {
#pragma unroll
            for (int t = 0; t < kMaxRows; ++t)
                if (t < T) acc[t] *= f_s[t];
            const int nk = min(256, k_end - c0);
            for (int kk = part; kk < nk; kk += nparts) {
                const size_t e = (size_t)(c0 + kk) * I + h * dh + pd;
                const float vv = DT ? bf2f(((const uint16_t*)a.v)[e]) : ((const float*)a.v)[e];
#pragma unroll
                for (int t = 0; t < kMaxRows; ++t)
                    if (t < T) acc[t] += S[t * 256 + kk] * vv;
            }
        }
        __syncthreads();
    }
    if (part < nparts) {
#pragma unroll
        for (int t = 0; t < kMaxRows; ++t)
            if (t < T) red[(part * T + t) * dh + pd] = acc[t];
    }
    __syncthreads();
    for (int i = tid; i < T * dh; i += 256) {
        const int t = i / dh, d = i % dh;
        float o = 0.f;
        for (int p = 0; p < nparts; ++p) o += red[(p * T + t) * dh + d];
        if (a.splits == 1)
            a.out[(size_t)t * I + h * dh + d] = o / l_s[t];
        else
            a.part_o[((size_t)sp * T + t) * I + h * dh + d] = o;
    }
    if (a.splits > 1 && tid < T) {
        float* ml = a.part_ml + (((size_t)sp * T + tid) * a.heads + h) * 2;
        ml[0] = m_s[tid];
        ml[1] = l_s[tid];
    }
}

__global__ __launch_bounds__(256) void attn_merge_kernel(const AttnArgs a) {
    const int t = blockIdx.x, I = a.i_dim;
    for (int n = threadIdx.x; n < I; n += 256) {
        const int h = n / a.d_head;
        float M = -INFINITY;
        for (int sp = 0; sp < a.splits; ++sp) M = fmaxf(M, a.part_ml[(((size_t)sp * a.T + t) * a.heads + h) * 2]);
        float L = 0.f, O = 0.f;
        for (int sp = 0; sp < a.splits; ++sp) {
            const float* ml = a.part_ml + (((size_t)sp * a.T + t) * a.heads + h) * 2;
            const float w = (ml[0] == -INFINITY) ? 0.f : expf(ml[0] - M);
            L += ml[1] * w;
            O += a.part_o[((size_t)sp * a.T + t) * I + n] * w;
        }
        a.out[(size_t)t * I + n] = O / L;
    }
}

hipError_t launch_attention(const AttnArgs& a, int dtype, hipStream_t st) {
    if (hipError_t e = raise_lds_limits(); e != hipSuccess) return e;
    const int nparts = 256 / a.d_head;
    const size_t smem = sizeof(float) * ((size_t)a.T * a.d_head + (size_t)a.T * 256 + 3 * kMaxRows +
                                         (size_t)nparts * a.T * a.d_head);
    const dim3 grid(a.heads, a.splits);
    if (dtype)
        hipLaunchKernelGGL(attn_kernel<1>, grid, dim3(256), smem, st, a);
    else
        hipLaunchKernelGGL(attn_kernel<0>, grid, dim3(256), smem, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.splits == 1) return e;
    hipLaunchKernelGGL(attn_merge_kernel, dim3(a.T), dim3(256), 0, st, a);
    return hipGetLastError();
}

// =====================================================================================
// Embedding gather from the tiled matrix (+ sinusoidal position).
// =====================================================================================
template <int DT>
__global__ __launch_bounds__(256) void embed_kernel(const EmbedArgs a) {
    constexpr int KT = DT ? 32 : 16, PL = KT / 4;
    const int t = blockIdx.x;
    const int base = (a.base_ptr ? *a.base_ptr : 0) + a.base_add;
    const int tok = a.tokens[base + t];
    const int row = (int)(((long long)tok + a.tie_shift) % a.vocab);
    const int pos = base + t;
    const double lg = log2(10000.0);
    for (int k = threadIdx.x; k < a.d; k += 256) {
        const size_t tile = (size_t)(row >> 4) * a.E.tk + (k / KT);
        const int ln = (row & 15) + 16 * ((k % KT) / PL), j = k % PL;
        const char* p = (const char*)a.E.w + tile * kTileBytes + ln * 16;
        float v = DT ? bf2f(((const uint16_t*)p)[j]) : ((const float*)p)[j];
        v *= a.embed_scale;
        if (a.sinusoidal) {
            const double ang = (double)pos * exp2(-(double)(2 * (k >> 1)) / (double)a.d * lg);
            v += (float)((k & 1) ? cos(ang) : sin(ang));
        }
        a.x[(size_t)t * a.d + k] = v;
    }
}

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
// =====================================================================================
__global__ __launch_bounds__(256) void finish_kernel(const FinishArgs a) {
    __shared__ float rm[kMaxRows], rsum[kMaxRows];
    __shared__ int ridx[kMaxRows];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    Ctl* c = a.ctl;
    if (a.mode != 3) {
        for (int t = wave; t < a.T; t += 4) {
            Stat r = stat_neutral();
            for (int p = lane; p < a.nparts; p += 64) {
                const StatPart sp = a.part[(size_t)p * kMaxRows + a.row_off + t];
                r = stat_merge(r, Stat{sp.m, sp.s, sp.idx});
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) r = stat_merge(r, stat_shfl_xor(r, o));
            if (lane == 0) {
                rm[t] = r.m;
                rsum[t] = r.s;
                ridx[t] = r.idx;
            }
        }
    }
    __syncthreads();
    if (tid != 0) return;
    const int w = a.which;
    if (a.mode == 3) {
        c->len[w] += a.rows_consumed;
        return;
    }
    for (int t = 0; t < a.T; ++t) c->res_rowtok[t] = ridx[t];
    if (a.mode == 0 || a.mode == 2) {
        const int tok = ridx[a.T - 1];
        const float pmax = 1.f / rsum[a.T - 1];
        const int pending = c->y_len - c->draft_start;
        const bool low = (a.mode == 0) && (pmax < a.alpha);
        const bool forced = (a.mode == 0) && c->n_max > 0 && pending >= c->n_max;
        const bool fb = low || forced;
        c->len[w] += a.rows_consumed;
        if (!fb && c->y_len < a.y_cap) {
            a.y[c->y_len] = tok;
            c->y_len += 1;
            if (a.mode == 2) c->draft_start = c->y_len;
        }
        c->res_tok = tok;
        c->res_flag = (fb ? 1 : 0) | ((forced && !low) ? 2 : 0);
        c->res_pmax = pmax;
        return;
    }
    // review of n = T - 1 drafts
    const int n = a.T - 1;
    int r = n;
    for (int i = 0; i < n; ++i) {
        const float nll = (rm[i] + logf(rsum[i])) - a.zt[a.row_off + i];
        c->res_nll[i] = nll;
        if (r == n && nll > a.alpha) r = i;
    }
    const int tok = ridx[r];
    const int ds = c->draft_start;
    a.y[ds + r] = tok;
    c->y_len = ds + r + 1;
    c->len[1] = c->y_len - 1;
    c->len[0] = min(c->len[0], c->y_len - 1);
    c->draft_start = c->y_len;
    c->res_r = r;
    c->res_n = n;
    c->res_tok = tok;
    c->res_pmax = 1.f / rsum[r];
    c->res_flag = 0;
}

hipError_t launch_finish(const FinishArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace bild
