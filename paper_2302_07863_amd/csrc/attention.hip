// KV-cache attention of the BiLD decoding path for gfx950 (see the banner below); launched as attn_kernel (up to
// 32 query rows, optional key splits), attn_rows_kernel (more query rows: encoder, prompt prefill) and
// attn_merge_kernel (joins key splits).
#include "kernel_common.h"

namespace bild {

constexpr int kAttnLdsLimit = 160 * 1024;

// =====================================================================================
// KV-cache attention on the matrix cores.  K is stored [position][I]; V is stored
// transposed, [I][capacity], so that both products contract over a contiguous axis:
//   S^T[key][row] = K[key][:] . q[row][:]      A = K tile (16 keys x 32 dims), B = q^T
//   O^T[dim][row] += V^T[dim][key] P[key][row] A = V^T tile (16 dims x 32 keys), B = P
// One workgroup per (head, key split); its waves take 32-key blocks round robin and keep
// a running (max, sum, O) per query row, merged across waves in LDS at the end.  The score
// tile leaves the MFMA with lane (row, g) holding keys 4g..4g+3 of each 16-key tile, which
// is exactly the B-operand order of the second product if its contraction index 8g+j is
// read as "key 4g+j of the first tile (j<4) / of the second tile (j>=4)" - so the
// probabilities never move between lanes; the V^T loads follow the same key order.
// q and P are real-valued: bf16 models split them into high and low bf16 parts.
// Cache rows beyond the valid length are finite (zero-filled at allocation, or stale
// values of discarded tokens), so a probability of exactly 0 removes them.
// =====================================================================================
// Hot arguments (see BILD_GEMM_HOT_PARAMS in gemm_body.h): what the first requests of an attention workgroup depend on,
// passed a second time as leading scalar parameters that arrive in scalar registers at wave start.
//   h_q, h_k, h_v, h_len   q, k, v, len_ptr
//   h_T                    T
//   h_p0                   heads | nw << 8 | causal << 12 | d_head << 13 | splits << 22 | log2(splits) << 29 (a power of two)
//   h_idim, h_vcap, h_badd, h_nkf   i_dim, vcap, base_add, nkeys_fixed
#define BILD_ATTN_HOT_PARAMS                                                                                   \
    const float* __restrict__ h_q, const void* __restrict__ h_k, const void* __restrict__ h_v,                 \
        const int* __restrict__ h_len, const int h_T, const int h_p0, const int h_idim, const int h_vcap,      \
        const int h_badd, const int h_nkf
#define BILD_ATTN_HOT_NAMES h_q, h_k, h_v, h_len, h_T, h_p0, h_idim, h_vcap, h_badd, h_nkf
__device__ __forceinline__ AttnArgs attn_hot(const AttnArgs& a, BILD_ATTN_HOT_PARAMS) {
    AttnArgs b = a;
    b.q = h_q; b.k = h_k; b.v = h_v; b.len_ptr = h_len; b.T = h_T;
    b.heads = h_p0 & 255; b.nw = (h_p0 >> 8) & 15; b.causal = (h_p0 >> 12) & 1; b.d_head = (h_p0 >> 13) & 511; b.splits = (h_p0 >> 22) & 127; b.lsplits = (h_p0 >> 29) & 7;
    b.i_dim = h_idim; b.vcap = h_vcap; b.base_add = h_badd; b.nkeys_fixed = h_nkf;
    return b;
}
static inline int attn_hot_p0(const AttnArgs& a) {
    int ls = 0;
    while ((1 << ls) < a.splits) ++ls;
    return a.heads | (a.nw << 8) | ((a.causal ? 1 : 0) << 12) | (a.d_head << 13) | (a.splits << 22) | (int)((unsigned)ls << 29);
}
#define BILD_ATTN_HOT(a)                                                                                             \
    (a).q, (a).k, (a).v, (a).len_ptr, (a).T,                                                                          \
        attn_hot_p0(a), (a).i_dim, \
        (a).vcap, (a).base_add, (a).nkeys_fixed

// FUSE: the finished output of the head stays in LDS (in q's place, in q's operand layout) for the output projection
// that the same workgroup runs next (attn_proj_kernel); nothing is written to memory here.
// `h`, `sp`: head and key split of this workgroup; `extra` runs right behind the first K/V request (attn_proj_kernel
// requests its weight tiles there).
template <int DT, int DH32, bool REL = false, bool FUSE = false, class Extra>
__device__ __forceinline__ void attn_body(const AttnArgs& a, const int h, const int sp, char* smem, Extra&& extra) {
    constexpr int DHP = DH32 * 32;   // head dim padded to the k-step of the first product
    constexpr int DT16 = DH32 * 2;   // 16-wide output tiles along the head dim
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform by construction
    const int nw = a.nw, nthr = nw << 6;  // (the launch has 64 * nw threads)
    const int T = a.T, dh = a.d_head, I = a.i_dim;
    const int NT = (T + 15) >> 4;
    const int tok_l = lane & 15, g = lane >> 4;
    const int qstride = DT ? (DHP + 8) * 2 : (DHP + 4) * 4;
    char* q_hi = smem;
    char* q_lo = smem + NT * 16 * qstride;  // bf16 only
    char* comb = smem + NT * 16 * qstride * (DT ? 2 : 1);
    float* cm = (float*)comb;                 // [nw][32]
    float* cl = cm + nw * 32;                 // [nw][32]
    f32x4* co = (f32x4*)(cl + nw * 32);       // [nw][NT][DT16][64]
    // relative-position models: this head's row of the bias table, [2*rel_d + 1], behind the merge buffers
    float* relb = REL ? (float*)(co + nw * NT * DT16 * 64) : nullptr;
    const int nrel = REL ? 2 * a.rel_d + 1 : 1;

    // One unconditional scalar load of the length (the launcher guarantees the pointer): it is requested here and
    // first used behind q's vector loads, so the two trips to memory overlap.
    const int len_v = *a.len_ptr;
    int base = 0, nkeys = 0, blk_begin = 0, blk_end = 0;
    auto ranges = [&]() {
        base = a.causal ? len_v + a.base_add : 0;
        nkeys = a.causal ? base + T : (a.nkeys_fixed > 0 ? a.nkeys_fixed : len_v);
        const int nblk = (nkeys + 31) >> 5;
        const int bps = (nblk + a.splits - 1) >> a.lsplits;  // (the key splits are a power of two)
        blk_begin = min(nblk, sp * bps);
        blk_end = min(nblk, blk_begin + bps);
    };

    // ---- stage q * scale (zero padded to NT*16 rows x DHP dims) ----
    // The memory counter retires loads in issue order, so q (needed first, and warm) is requested before the first
    // K/V block: `hook` runs between the requests of the first round and their conversion.  The loads are
    // unconditional (clamped address, value selected afterwards), else they would be waited for where the branches join.
    auto stage_q = [&](auto&& hook) {
        const int npieces = NT * 16 * (DHP / 4);
        auto piece = [&](int i, auto&& hk) {
            const int t = i / (DHP / 4), d4 = (i % (DHP / 4)) * 4;
            const bool real = t < T && d4 < dh;
            float4 v = ld_act4(a.q + (size_t)min(t, T - 1) * I + h * dh + min(d4, dh - 4));
            __builtin_amdgcn_sched_barrier(0);  // q goes out before anything waits for the length (the hook's first use of it)
            hk();
            __builtin_amdgcn_sched_barrier(0);  // the conversion of q stays behind the K/V requests
            v.x = real ? v.x * a.scale : 0.f; v.y = real ? v.y * a.scale : 0.f;
            v.z = real ? v.z * a.scale : 0.f; v.w = real ? v.w * a.scale : 0.f;
            if (DT) {
                uint32_t h01, l01, h23, l23;
                split_bf16x2(v.x, v.y, h01, l01);
                split_bf16x2(v.z, v.w, h23, l23);
                *(uint2*)(q_hi + t * qstride + d4 * 2) = make_uint2(h01, h23);
                *(uint2*)(q_lo + t * qstride + d4 * 2) = make_uint2(l01, l23);
            } else {
                *(float4*)(q_hi + t * qstride + d4 * 4) = v;
            }
        };
        // a thread past the end redoes the last piece (same value to the same place), so that its load stays unconditional
        piece(min(tid, npieces - 1), hook);
        for (int i = tid + nthr; i < npieces; i += nthr) piece(i, [] {});
    };

    float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
    f32x4 O[2][DT16];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int dt = 0; dt < DT16; ++dt) O[nt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    const size_t esz = DT ? 2 : 4;
    constexpr int KN = DT ? DH32 : DH32 * 2, VN = DT ? 1 : 2;
    auto load_kv = [&](uint4 (&Kr)[2][KN], uint4 (&Vr)[DT16][VN], int blk) {
        const int key0 = blk * 32;
        // ---- loads: K rows of both 16-key tiles, V^T columns of the same 32 keys ----
#pragma unroll
        for (int ab = 0; ab < 2; ++ab) {
            const char* krow = (const char*)a.k + ((size_t)(key0 + ab * 16 + tok_l) * I + h * dh) * esz;
            if (DT) {
#pragma unroll
                for (int ks = 0; ks < DH32; ++ks) {
                    // dims past the head read a clamped (valid) address: q is zero there and the cache is finite
                    const int d0 = min(ks * 32 + g * 8, dh - 8);
                    Kr[ab][ks] = *(const uint4*)(krow + d0 * 2);
                }
            } else {
#pragma unroll
                for (int ks = 0; ks < DH32 * 2; ++ks) {
                    const int d0 = min(ks * 16 + g * 4, dh - 4);
                    Kr[ab][ks] = *(const uint4*)(krow + d0 * 4);
                }
            }
        }
#pragma unroll
        for (int dt = 0; dt < DT16; ++dt) {
            // output dims past the head are never stored: their V^T rows read a clamped (valid) row
            const int d = min(dt * 16 + tok_l, dh - 1);
            const char* vrow = (const char*)a.v + ((size_t)(h * dh + d) * a.vcap + key0 + g * 4) * esz;
            if (DT) {
                const uint2 va = *(const uint2*)vrow, vb = *(const uint2*)(vrow + 16 * 2);
                Vr[dt][0] = make_uint4(va.x, va.y, vb.x, vb.y);
            } else {
                Vr[dt][0] = *(const uint4*)vrow;
                Vr[dt][1] = *(const uint4*)(vrow + 16 * 4);
            }
        }
    };
    auto process = [&](uint4 (&Kr)[2][KN], uint4 (&Vr)[DT16][VN], int blk) {
        const int key0 = blk * 32;
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            if (nt >= NT) continue;
            const int t = nt * 16 + tok_l;
            // ---- scores of this row against the 32 keys ----
            f32x4 s[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
            if (DT) {
#pragma unroll
                for (int ks = 0; ks < DH32; ++ks) {
                    const bf16x8 Bh = __builtin_bit_cast(bf16x8, *(const uint4*)(q_hi + t * qstride + (ks * 32 + g * 8) * 2));
                    const bf16x8 Bl = __builtin_bit_cast(bf16x8, *(const uint4*)(q_lo + t * qstride + (ks * 32 + g * 8) * 2));
#pragma unroll
                    for (int ab = 0; ab < 2; ++ab) {
                        const bf16x8 Ak = __builtin_bit_cast(bf16x8, Kr[ab][ks]);
                        s[ab] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Ak, Bh, s[ab], 0, 0, 0);
                        s[ab] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Ak, Bl, s[ab], 0, 0, 0);
                    }
                }
            } else {
#pragma unroll
                for (int ks = 0; ks < DH32 * 2; ++ks) {
                    const float4 b = *(const float4*)(q_hi + t * qstride + (ks * 16 + g * 4) * 4);
                    const float bb[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
                    for (int ab = 0; ab < 2; ++ab) {
                        const float aa[4] = {__uint_as_float(Kr[ab][ks].x), __uint_as_float(Kr[ab][ks].y),
                                             __uint_as_float(Kr[ab][ks].z), __uint_as_float(Kr[ab][ks].w)};
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            s[ab] = __builtin_amdgcn_mfma_f32_16x16x4f32(aa[j], bb[j], s[ab], 0, 0, 0);
                    }
                }
            }
            // ---- mask, running max / sum ----
            const int lim = a.causal ? min(nkeys - 1, base + t) : nkeys - 1;  // last visible key of this row
            float tmax = -INFINITY;
#pragma unroll
            for (int ab = 0; ab < 2; ++ab)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int key = key0 + ab * 16 + g * 4 + v;
                    if constexpr (REL) {
                        // learned bias of the clamped signed distance key - query, one row of the table per head;
                        // the clamp keeps the index inside the table for padded rows and keys past the end as well
                        const int qpos = (a.causal ? base : a.base_add) + t;
                        const int dist = max(-a.rel_d, min(a.rel_d, key - qpos));
                        s[ab][v] += relb[a.rel_d + dist];
                    }
                    if (key > lim || t >= T) s[ab][v] = -INFINITY;
                    tmax = fmaxf(tmax, s[ab][v]);
                }
            tmax = quad_rows_max(tmax);
            const float m_new = fmaxf(m_run[nt], tmax);
            const float f = (m_run[nt] == -INFINITY) ? 0.f : fexp(m_run[nt] - m_new);
            float p[2][4], psum = 0.f;
#pragma unroll
            for (int ab = 0; ab < 2; ++ab)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    p[ab][v] = (m_new == -INFINITY) ? 0.f : fexp(s[ab][v] - m_new);
                    psum += p[ab][v];
                }
            psum = quad_rows_sum(psum);
            l_run[nt] = l_run[nt] * f + psum;
            m_run[nt] = m_new;
            // ---- O = O * f + V^T P ----
            if (DT) {
                uint32_t ph[4], pl[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) split_bf16x2(p[j >> 1][(j & 1) * 2], p[j >> 1][(j & 1) * 2 + 1], ph[j], pl[j]);
                const bf16x8 Ph = __builtin_bit_cast(bf16x8, make_uint4(ph[0], ph[1], ph[2], ph[3]));
                const bf16x8 Pl = __builtin_bit_cast(bf16x8, make_uint4(pl[0], pl[1], pl[2], pl[3]));
#pragma unroll
                for (int dt = 0; dt < DT16; ++dt) {
                    O[nt][dt] *= f;
                    const bf16x8 Av = __builtin_bit_cast(bf16x8, Vr[dt][0]);
                    O[nt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Av, Ph, O[nt][dt], 0, 0, 0);
                    O[nt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Av, Pl, O[nt][dt], 0, 0, 0);
                }
            } else {
#pragma unroll
                for (int dt = 0; dt < DT16; ++dt) {
                    O[nt][dt] *= f;
#pragma unroll
                    for (int ab = 0; ab < 2; ++ab) {
                        const uint4 vv = Vr[dt][DT ? 0 : ab];
                        const float aa[4] = {__uint_as_float(vv.x), __uint_as_float(vv.y), __uint_as_float(vv.z),
                                             __uint_as_float(vv.w)};
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            O[nt][dt] = __builtin_amdgcn_mfma_f32_16x16x4f32(aa[j], p[ab][j], O[nt][dt], 0, 0, 0);
                    }
                }
            }
        }
    };
    // two register buffers: the next 32-key block loads while the current one is processed
    {
        uint4 K0[2][KN], V0[DT16][VN];
        int blk = 0;
        // a wave without a block requests block 0 of the cache all the same (valid memory, never processed): the
        // request sits between q's loads and their use and must not be conditional
        // The bias row is requested ahead of q and stored with it, so that its store does not wait for the K/V block
        // requested in between.  A one-wave workgroup needs several pieces per thread for the row: RP of them are requested
        // together (a loop of load-then-store would pay one trip to memory per piece); indices past the end are clamped, so
        // such a thread rewrites the last entry with its own value.
        constexpr int RP = 8;
        float relv[RP];
        if constexpr (REL) {
#pragma unroll
            for (int p = 0; p < RP; ++p) relv[p] = a.rel_bias[h * nrel + min(tid + p * nthr, nrel - 1)];
        }
        stage_q([&] {
            ranges();
            blk = blk_begin + wave;
            load_kv(K0, V0, blk < blk_end ? blk : 0);
            extra();
        });
        if constexpr (REL) {
#pragma unroll
            for (int p = 0; p < RP; ++p) relb[min(tid + p * nthr, nrel - 1)] = relv[p];
            for (int i = tid + RP * nthr; i < nrel; i += nthr) relb[i] = a.rel_bias[h * nrel + i];
        }
        __syncthreads();
        if constexpr (DH32 <= 2) {
            uint4 K1[2][KN], V1[DT16][VN];
            for (; blk < blk_end; blk += 2 * nw) {
                if (blk + nw < blk_end) load_kv(K1, V1, blk + nw);
                process(K0, V0, blk);
                if (blk + nw >= blk_end) break;
                if (blk + 2 * nw < blk_end) load_kv(K0, V0, blk + 2 * nw);
                process(K1, V1, blk + nw);
            }
        } else {  // 128-wide heads: one buffer, the registers are needed for the output tiles
            for (; blk < blk_end; blk += nw) {
                process(K0, V0, blk);
                if (blk + nw < blk_end) load_kv(K0, V0, blk + nw);
            }
        }
    }
    // ---- merge the waves' partial results ----
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        if (nt >= NT) continue;
        if (g == 0) {
            cm[wave * 32 + nt * 16 + tok_l] = m_run[nt];
            cl[wave * 32 + nt * 16 + tok_l] = l_run[nt];
        }
#pragma unroll
        for (int dt = 0; dt < DT16; ++dt) co[((wave * NT + nt) * DT16 + dt) * 64 + lane] = O[nt][dt];
    }
    __syncthreads();
    for (int qd = wave; qd < NT * DT16; qd += nw) {
        const int nt = qd / DT16, dt = qd % DT16;
        const int t = nt * 16 + tok_l, d0 = dt * 16 + g * 4;
        // The waves' results are joined in the order of the waves.  With four waves (the usual workgroup) the reads go out
        // together; a loop over a run-time count would wait for each wave's values before asking for the next.
        float M = -INFINITY, Lsum = 0.f;
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
        if (nw == 4) {
            float mw[4], lw[4];
            f32x4 ow[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                mw[w] = cm[w * 32 + nt * 16 + tok_l];
                lw[w] = cl[w * 32 + nt * 16 + tok_l];
                ow[w] = co[((w * NT + nt) * DT16 + dt) * 64 + lane];
            }
#pragma unroll
            for (int w = 0; w < 4; ++w) M = fmaxf(M, mw[w]);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float wgt = (mw[w] == -INFINITY) ? 0.f : fexp(mw[w] - M);
                Lsum += lw[w] * wgt;
                acc += ow[w] * wgt;
            }
        } else {
            for (int w = 0; w < nw; ++w) M = fmaxf(M, cm[w * 32 + nt * 16 + tok_l]);
            for (int w = 0; w < nw; ++w) {
                const float mw = cm[w * 32 + nt * 16 + tok_l];
                const float wgt = (mw == -INFINITY) ? 0.f : fexp(mw - M);
                Lsum += cl[w * 32 + nt * 16 + tok_l] * wgt;
                acc += co[((w * NT + nt) * DT16 + dt) * 64 + lane] * wgt;
            }
        }
        if constexpr (FUSE) {
            const float inv = t < T ? 1.f / Lsum : 0.f;
            const float o0 = t < T ? acc[0] * inv : 0.f, o1 = t < T ? acc[1] * inv : 0.f;
            const float o2 = t < T ? acc[2] * inv : 0.f, o3 = t < T ? acc[3] * inv : 0.f;
            if (DT) {
                uint32_t h01, l01, h23, l23;
                split_bf16x2(o0, o1, h01, l01);
                split_bf16x2(o2, o3, h23, l23);
                *(uint2*)(q_hi + t * qstride + d0 * 2) = make_uint2(h01, h23);
                *(uint2*)(q_lo + t * qstride + d0 * 2) = make_uint2(l01, l23);
            } else {
                *(float4*)(q_hi + t * qstride + d0 * 4) = make_float4(o0, o1, o2, o3);
            }
        } else if (t < T && d0 < dh) {
            if (a.splits == 1) {
                const float inv = 1.f / Lsum;
                if (DT && a.ob_hi) {
                    uint32_t h01, l01, h23, l23;
                    split_bf16x2(acc[0] * inv, acc[1] * inv, h01, l01);
                    split_bf16x2(acc[2] * inv, acc[3] * inv, h23, l23);
                    st_u64(a.ob_hi + (size_t)t * I + h * dh + d0, h01, h23);
                    st_u64(a.ob_lo + (size_t)t * I + h * dh + d0, l01, l23);
                } else {
                    st_act4(a.out + (size_t)t * I + h * dh + d0, make_float4(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv));
                }
            } else {
                st_act4(a.part_o + ((size_t)sp * T + t) * I + h * dh + d0, make_float4(acc[0], acc[1], acc[2], acc[3]));
                if (dt == 0 && g == 0) {
                    float* ml = a.part_ml + (((size_t)sp * T + t) * a.heads + h) * 2;
                    st_act(ml, M);
                    st_act(ml + 1, Lsum);
                }
            }
        }
    }
}

template <int DT, int DH32, bool REL = false>
__global__ __launch_bounds__(512) void attn_kernel(BILD_ATTN_HOT_PARAMS, const AttnArgs a0) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const AttnArgs a = attn_hot(a0, BILD_ATTN_HOT_NAMES);
    attn_body<DT, DH32, REL>(a, (int)blockIdx.x, (int)blockIdx.y, smem, [] {});  // grid: heads x key splits
}

// More than kMaxRows query rows: blockIdx.z picks the block of rows (key splits are not combined with it).
template <int DT, int DH32, bool REL = false>
__global__ __launch_bounds__(512) void attn_rows_kernel(BILD_ATTN_HOT_PARAMS, const AttnArgs a0) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const AttnArgs a = attn_hot(a0, BILD_ATTN_HOT_NAMES);
    AttnArgs b = a;
    const int r0 = (int)blockIdx.z * kMaxRows;
    b.T = min(kMaxRows, a.T - r0);
    b.q = a.q + (size_t)r0 * a.i_dim;
    b.out = a.out + (size_t)r0 * a.i_dim;
    b.base_add = a.base_add + r0;
    attn_body<DT, DH32, REL>(b, (int)blockIdx.x, 0, smem, [] {});
}

// Attention of one head followed by that head's share of the output projection, for single-row passes of the narrow
// models: workgroup (head h, column group c) runs the whole attention of head h (every column group repeats it: the
// cache of a head is a few KiB to 128 KiB) and multiplies the result by the rows h * d_head .. of W_o for its
// share of the output features.  The product is a partial result of the residual update, one per head
// (proj_out[h][t][n]); the projection that reads the residual stream next adds them up while staging, so the
// output projection costs no launch of its own.  The weight tiles are requested at entry and arrive during the attention.
template <int DT, int DH32, bool REL = false>
__global__ __launch_bounds__(512) void attn_proj_kernel(BILD_ATTN_HOT_PARAMS, const AttnArgs a0) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const AttnArgs a = attn_hot(a0, BILD_ATTN_HOT_NAMES);
    constexpr int KT = DT ? 32 : 16, DHP = DH32 * 32, KH = DHP / KT, MAXN = DT ? 4 : 2;  // (fp32: four input tiles per head already)
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), nw = a.nw;
    const int h = (int)blockIdx.x, c = (int)blockIdx.y;
    // Everything about W_o is read from the argument structure, which is not among the values that arrive in registers:
    // it is first touched behind the first K/V request (the barrier keeps the compiler from moving the division up, which
    // would make the kernel start with a wait for the structure).
    int npc = 0, khr = 0, kt0 = 0;
    uint4 Wt[MAXN][KH];
    auto request_w = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        npc = (a.wo.tn + a.cgroups - 1) / a.cgroups;  // feature tiles per column group (grid: heads x cgroups)
        khr = a.d_head / KT;                           // this head's input tiles (d_head is a multiple of KT)
        kt0 = h * khr;
#pragma unroll
        for (int i = 0; i < MAXN; ++i) {
            const int n = min(c * npc + wave + i * nw, a.wo.tn - 1);
#pragma unroll
            for (int j = 0; j < KH; ++j)
                Wt[i][j] = *(const uint4*)((const char*)a.wo.w + ((size_t)n * a.wo.tk + kt0 + min(j, khr - 1)) * kTileBytes + lane * 16);
        }
    };
    attn_body<DT, DH32, REL, true>(a, h, 0, smem, request_w);
    __syncthreads();
    const int tok_l = lane & 15, g = lane >> 4;
    const int qstride = DT ? (DHP + 8) * 2 : (DHP + 4) * 4;
    const int NT = (a.T + 15) >> 4;
    const char* o_hi = smem;
    const char* o_lo = smem + NT * 16 * qstride;
#pragma unroll
    for (int i = 0; i < MAXN; ++i) {
        const int n = c * npc + wave + i * nw;  // wave-uniform
        if (n >= (c + 1) * npc || n >= a.wo.tn) continue;
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f}, acc2 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < KH; ++j) {
            if (j >= khr) continue;
            if (DT) {
                const bf16x8 Aw = __builtin_bit_cast(bf16x8, Wt[i][j]);
                const bf16x8 Bh = __builtin_bit_cast(bf16x8, *(const uint4*)(o_hi + tok_l * qstride + (j * 32 + g * 8) * 2));
                const bf16x8 Bl = __builtin_bit_cast(bf16x8, *(const uint4*)(o_lo + tok_l * qstride + (j * 32 + g * 8) * 2));
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Aw, Bh, acc, 0, 0, 0);
                acc2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Aw, Bl, acc2, 0, 0, 0);
            } else {
                const float4 b = *(const float4*)(o_hi + tok_l * qstride + (j * 16 + g * 4) * 4);
                const float aa[4] = {__uint_as_float(Wt[i][j].x), __uint_as_float(Wt[i][j].y), __uint_as_float(Wt[i][j].z),
                                     __uint_as_float(Wt[i][j].w)};
                const float bb[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
                for (int v = 0; v < 4; v += 2) {
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(aa[v], bb[v], acc, 0, 0, 0);
                    acc2 = __builtin_amdgcn_mfma_f32_16x16x4f32(aa[v + 1], bb[v + 1], acc2, 0, 0, 0);
                }
            }
        }
        acc += acc2;
        if (tok_l < a.T)
            st_act4(a.proj_out + (size_t)h * a.proj_stride + (size_t)tok_l * a.d_model + n * 16 + g * 4,
                    make_float4(acc[0], acc[1], acc[2], acc[3]));
    }
}

// Joins the key splits of attention: out[t][n] = sum_s w_s O_s[t][n] / sum_s w_s L_s with w_s = exp(m_s - max m) of
// (row t, head of n).  Unit `u` covers 256 float4 pieces of the [T][I] output; every thread owns one piece and issues
// the loads of all splits together (eight at a time).
__device__ __forceinline__ void attn_merge_body(const AttnArgs& a, const int u) {
    const int I = a.i_dim, n4 = I >> 2;
    const int e = u * 256 + (int)threadIdx.x;
    if (threadIdx.x >= 256 || e >= a.T * n4) return;
    const int t = e / n4, n = (e - t * n4) * 4;
    const int h = n / a.d_head;
    const size_t ml_stride = (size_t)a.T * a.heads * 2, o_stride = (size_t)a.T * I;
    const float* ml = a.part_ml + ((size_t)t * a.heads + h) * 2;
    const float* op = a.part_o + (size_t)t * I + n;
    float M = -INFINITY;
    for (int s0 = 0; s0 < a.splits; s0 += 8) {
        float m[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) m[k] = ld_act(ml + min(s0 + k, a.splits - 1) * ml_stride);
#pragma unroll
        for (int k = 0; k < 8; ++k) M = fmaxf(M, m[k]);
    }
    float L = 0.f;
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s0 = 0; s0 < a.splits; s0 += 8) {
        float m[8], l[8];
        float4 o[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int sc = min(s0 + k, a.splits - 1);
            m[k] = ld_act(ml + sc * ml_stride);
            l[k] = ld_act(ml + sc * ml_stride + 1);
            o[k] = ld_act4(op + sc * o_stride);
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float w = (s0 + k < a.splits && m[k] != -INFINITY) ? expf(m[k] - M) : 0.f;
            L += l[k] * w;
            r.x += o[k].x * w; r.y += o[k].y * w; r.z += o[k].z * w; r.w += o[k].w * w;
        }
    }
    const float inv = 1.f / L;
    if (a.ob_hi) {
        uint32_t h01, l01, h23, l23;
        split_bf16x2(r.x * inv, r.y * inv, h01, l01);
        split_bf16x2(r.z * inv, r.w * inv, h23, l23);
        st_u64(a.ob_hi + (size_t)t * I + n, h01, h23);
        st_u64(a.ob_lo + (size_t)t * I + n, l01, l23);
    } else {
        st_act4(a.out + (size_t)t * I + n, make_float4(r.x * inv, r.y * inv, r.z * inv, r.w * inv));
    }
}

__global__ __launch_bounds__(256) void attn_merge_kernel(const AttnArgs a) { attn_merge_body(a, (int)blockIdx.x); }

size_t attn_lds_bytes(int dtype, int d_head, int T, int nw) {
    const int dh32 = d_head <= 32 ? 1 : (d_head <= 64 ? 2 : 4), dhp = dh32 * 32, nt = (T + 15) / 16;
    const size_t q = (size_t)nt * 16 * (dtype ? (dhp + 8) * 2 * 2 : (dhp + 4) * 4);
    return q + (size_t)nw * 32 * 4 * 2 + (size_t)nw * nt * (dh32 * 2) * 64 * 16;
}

// The attention kernels may ask for more than the default 64 KiB of dynamic LDS.
static hipError_t attn_raise_lds_limits() {
    static hipError_t done = [] {
        const void* fns[] = {
                             (const void*)attn_rows_kernel<0, 1>, (const void*)attn_rows_kernel<0, 2>,
                             (const void*)attn_rows_kernel<0, 4>, (const void*)attn_rows_kernel<1, 1>,
                             (const void*)attn_rows_kernel<1, 2>, (const void*)attn_rows_kernel<1, 4>,
                             (const void*)attn_kernel<0, 1>, (const void*)attn_kernel<0, 2>,
                             (const void*)attn_kernel<0, 4>, (const void*)attn_kernel<1, 1>,
                             (const void*)attn_kernel<1, 2>, (const void*)attn_kernel<1, 4>,
                             (const void*)attn_rows_kernel<0, 1, true>, (const void*)attn_rows_kernel<0, 2, true>,
                             (const void*)attn_rows_kernel<0, 4, true>, (const void*)attn_rows_kernel<1, 1, true>,
                             (const void*)attn_rows_kernel<1, 2, true>, (const void*)attn_rows_kernel<1, 4, true>,
                             (const void*)attn_kernel<0, 1, true>, (const void*)attn_kernel<0, 2, true>,
                             (const void*)attn_kernel<0, 4, true>, (const void*)attn_kernel<1, 1, true>,
                             (const void*)attn_kernel<1, 2, true>, (const void*)attn_kernel<1, 4, true>,
                             (const void*)attn_proj_kernel<0, 1>, (const void*)attn_proj_kernel<0, 2>,
                             (const void*)attn_proj_kernel<1, 1>, (const void*)attn_proj_kernel<1, 2>,
                             (const void*)attn_proj_kernel<0, 1, true>, (const void*)attn_proj_kernel<0, 2, true>,
                             (const void*)attn_proj_kernel<1, 1, true>, (const void*)attn_proj_kernel<1, 2, true>};
        for (const void* f : fns) {
            hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kAttnLdsLimit);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }();
    return done;
}

hipError_t attention_init() { return attn_raise_lds_limits(); }

hipError_t launch_attention_proj(const AttnArgs& a, int dtype, hipStream_t st) {
    if (hipError_t e = attn_raise_lds_limits(); e != hipSuccess) return e;
    const int kt = dtype ? 32 : 16;
    const int dh32 = a.d_head <= 32 ? 1 : (a.d_head <= 64 ? 2 : 4);
    if (a.T < 1 || a.T > 16 || a.splits != 1 || !a.len_ptr || !a.wo.w || !a.proj_out || a.cgroups < 1 || a.d_head % kt || a.d_head > 64 ||
        a.wo.k != a.heads * a.d_head || a.wo.n != a.d_model || (a.rel_bias && a.rel_d < 1))
        return hipErrorInvalidValue;
    if (a.heads > 255 || a.nw > 15) return hipErrorInvalidValue;  // (BILD_ATTN_HOT packs them)
    const int npc = (a.wo.tn + a.cgroups - 1) / a.cgroups;
    if ((npc + a.nw - 1) / a.nw > (dtype ? 4 : 2)) return hipErrorInvalidValue;  // feature tiles a wave keeps in registers
    const size_t smem = attn_lds_bytes(dtype, a.d_head, a.T, a.nw) + (a.rel_bias ? (size_t)(2 * a.rel_d + 1) * 4 : 0);
    if (smem > (size_t)kAttnLdsLimit) return hipErrorInvalidValue;
    const dim3 grid(a.heads, a.cgroups), block(64 * a.nw);
#define BILD_AP(DTV, DHV)                                                                       \
    do {                                                                                        \
        if (a.rel_bias) hipLaunchKernelGGL((attn_proj_kernel<DTV, DHV, true>), grid, block, smem, st, BILD_ATTN_HOT(a), a); \
        else hipLaunchKernelGGL((attn_proj_kernel<DTV, DHV>), grid, block, smem, st, BILD_ATTN_HOT(a), a);        \
    } while (0)
    if (dtype) {
        if (dh32 == 1) BILD_AP(1, 1); else BILD_AP(1, 2);
    } else {
        if (dh32 == 1) BILD_AP(0, 1); else BILD_AP(0, 2);
    }
#undef BILD_AP
    return hipGetLastError();
}

hipError_t launch_attention(const AttnArgs& a, int dtype, hipStream_t st) {
    if (hipError_t e = attn_raise_lds_limits(); e != hipSuccess) return e;
    const int dh32 = a.d_head <= 32 ? 1 : (a.d_head <= 64 ? 2 : 4);
    const unsigned row_blocks = (unsigned)((a.T + kMaxRows - 1) / kMaxRows);
    if ((row_blocks > 1 && a.splits != 1) || !a.len_ptr) return hipErrorInvalidValue;
    if (a.heads > 255 || a.nw > 15 || a.d_head > 511 || a.splits < 1 || a.splits > 64 || (a.splits & (a.splits - 1))) return hipErrorInvalidValue;  // (BILD_ATTN_HOT packs them)
    if (a.rel_bias && a.rel_d < 1) return hipErrorInvalidValue;
    const size_t smem = attn_lds_bytes(dtype, a.d_head, std::min(a.T, kMaxRows), a.nw) +
                        (a.rel_bias ? (size_t)(2 * a.rel_d + 1) * 4 : 0);  // + one head's row of the bias table
    if (smem > (size_t)kAttnLdsLimit) return hipErrorInvalidValue;
    const dim3 grid(a.heads, a.splits, row_blocks), block(64 * a.nw);
#define BILD_ATTN(DTV, DHV)                                                                     \
    do {                                                                                        \
        if (row_blocks > 1 && a.rel_bias)                                                       \
            hipLaunchKernelGGL((attn_rows_kernel<DTV, DHV, true>), grid, block, smem, st, BILD_ATTN_HOT(a), a);   \
        else if (row_blocks > 1)                                                                \
            hipLaunchKernelGGL((attn_rows_kernel<DTV, DHV>), grid, block, smem, st, BILD_ATTN_HOT(a), a);         \
        else if (a.rel_bias)                                                                    \
            hipLaunchKernelGGL((attn_kernel<DTV, DHV, true>), grid, block, smem, st, BILD_ATTN_HOT(a), a);        \
        else                                                                                    \
            hipLaunchKernelGGL((attn_kernel<DTV, DHV>), grid, block, smem, st, BILD_ATTN_HOT(a), a);              \
    } while (0)
    if (dtype) {
        if (dh32 == 1) BILD_ATTN(1, 1); else if (dh32 == 2) BILD_ATTN(1, 2); else BILD_ATTN(1, 4);
    } else {
        if (dh32 == 1) BILD_ATTN(0, 1); else if (dh32 == 2) BILD_ATTN(0, 2); else BILD_ATTN(0, 4);
    }
#undef BILD_ATTN
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.splits == 1 || a.defer_merge) return e;
    hipLaunchKernelGGL(attn_merge_kernel, dim3((a.T * (a.i_dim / 4) + 255) / 256), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace bild
