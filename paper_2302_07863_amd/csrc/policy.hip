// Policy kernels of the BiLD library (gfx950): merge of the LM-head partial statistics, the fallback test
// (Section 3.3), the rollback test (Section 3.4), the commit of Algorithm 1 on the device, and the draws of the
// sampling variant (Appendix, "BiLD with Sampling") with the rejection-sampling acceptance of the methods the
// paper compares with (Section 4.2).
#include "kernel_common.h"

namespace bild {

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
constexpr int kFinishLds = 4 * kMaxRows * 4;
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
// nucleus_search finds the threshold key and the nucleus' mass (in units of exp(z - m)); weighted_walk draws.
__device__ __forceinline__ void nucleus_search(const float* __restrict__ z, int V, float m, float top_p, char* ws,
                                               uint32_t& K_out, float& mass_out) {
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
    K_out = K;
    mass_out = mass;
}

// Inverse-CDF draw over the ids of a row, walked in increasing id: the first id whose running weight exceeds
// u * total.  weight(i) >= 0 is the (unnormalised) probability of id i, the same for every thread; `total` < 0
// means "add the weights up here" (wave sums in wave order).  Returns the token to every thread.
template <class W>
__device__ __forceinline__ int weighted_walk(W weight, int V, float total, float u, char* ws) {
    float* bins = (float*)ws;              // [16 waves][16]
    float* tmass = bins + 16 * 16;         // [1024]
    float* sc = tmass + 1024;              // scalars
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nthr = blockDim.x, nwv = nthr >> 6;
    __syncthreads();                       // the workspace may still be read by an earlier search or walk
    // ---- every thread owns a run of consecutive ids ----
    const int chunk = (V + nthr - 1) / nthr;
    const int i0 = min(tid * chunk, V), i1 = min(i0 + chunk, V);
    float mine = 0.f;
    for (int i = i0; i < i1; ++i) mine += weight(i);
    tmass[tid] = mine;
    const float wsum = wave_sum(mine);
    if (lane == 0) bins[wave] = wsum;
    __syncthreads();
    if (tid == 0) {
        float mass = total;
        if (mass < 0.f) {
            mass = 0.f;
            for (int w = 0; w < nwv; ++w) mass += bins[w];
        }
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
            const float wi = weight(i);
            if (wi > 0.f) {
                last = i;
                run += wi;
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
            if (weight(i) > 0.f) best = max(best, i);
        for (int o = 32; o > 0; o >>= 1) best = max(best, __shfl_xor(best, o, 64));
        if (lane == 0) bins[wave] = __int_as_float(best);
        __syncthreads();
        for (int w = 0; w < nwv; ++w) tok = max(tok, __float_as_int(bins[w]));
    }
    return tok;
}

__device__ __forceinline__ int nucleus_draw(const float* __restrict__ z, int V, float m, float top_p, float u, char* ws) {
    uint32_t K;
    float mass;
    nucleus_search(z, V, m, top_p, ws, K, mass);
    return weighted_walk([&](int i) { const float zi = z[i]; return float_key(zi) >= K ? expf(zi - m) : 0.f; }, V, mass, u, ws);
}

// Merge of the LM-head partial statistics of the rows of a pass into (max, sum exp, argmax) per row, in LDS.  With at
// least as many waves as rows, every row gets nwv / T waves, each merging a contiguous share of the row's partials
// (lanes stride through it, eight loads in flight per lane), so that a single row with two thousand partials (250 112
// ids) costs one trip to memory instead of four; the shares are then joined in a fixed order.  More rows than waves: the
// rows are dealt to the waves.  Ends with a barrier.
__device__ __forceinline__ void merge_partials(const FinishArgs& a, float* rm, float* rsum, int* ridx) {
    __shared__ StatPart share[16];  // [row * wpr + share] (at most 16 waves)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwv = blockDim.x >> 6;
    auto merge_range = [&](int t, int p_begin, int p_end) {
        Stat r = stat_neutral();
        for (int p0 = p_begin + lane; p0 < p_end; p0 += 64 * 8) {
            StatPart sp[8];
#pragma unroll
            for (int k = 0; k < 8; ++k)
                sp[k] = a.part[(size_t)min(p0 + k * 64, p_end - 1) * kMaxRows + a.row_off + t];
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (p0 + k * 64 < p_end) r = stat_merge(r, Stat{sp[k].m, sp[k].s, sp[k].idx});
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) r = stat_merge(r, stat_shfl_xor(r, o));
        return r;
    };
    if (a.T <= nwv) {
        const int wpr = nwv / a.T;                      // waves per row
        const int per = (a.nparts + wpr - 1) / wpr;     // partials per share
        const int t = wave / wpr, c = wave - t * wpr;
        if (t < a.T) {
            const int p_begin = min(c * per, a.nparts), p_end = min(p_begin + per, a.nparts);
            const Stat r = merge_range(t, p_begin, p_end);  // (an empty share stays neutral)
            if (lane == 0) {
                StatPart sp;
                sp.m = r.m; sp.s = r.s; sp.idx = r.idx; sp.pad = 0;
                share[wave] = sp;
            }
        }
        __syncthreads();
        if (tid < a.T) {
            Stat r = stat_neutral();
            for (int c2 = 0; c2 < wpr; ++c2) {
                const StatPart sp = share[tid * wpr + c2];
                r = stat_merge(r, Stat{sp.m, sp.s, sp.idx});
            }
            rm[tid] = r.m;
            rsum[tid] = r.s;
            ridx[tid] = r.idx;
        }
    } else {
        for (int t = wave; t < a.T; t += nwv) {
            const Stat r = merge_range(t, 0, a.nparts);
            if (lane == 0) {
                rm[t] = r.m;
                rsum[t] = r.s;
                ridx[t] = r.idx;
            }
        }
    }
    __syncthreads();
}

// drawn_in >= 0: the token of the sampling variant, drawn before the call (finish_draw_kernel)
template <bool SAMPLE>
__device__ __forceinline__ void finish_body(const FinishArgs& a, char* lds, int drawn_in = -1) {
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
    if (a.mode != 3) merge_partials(a, rm, rsum, ridx);
    // Sampling variant: the token that will be committed is drawn by the whole workgroup from the row the
    // policy selects (the last row of a step; row r of a review), at the position it will occupy.
    int drawn = drawn_in;
    int r_given = -1;  // rejection-sampling acceptance: the index of the first refused draft (n: none), decided here
    if (SAMPLE && a.top_p > 0.f && a.mode <= 2) {
        int* sel = (int*)(lds + kFinishLds);  // [0] row, [1] position
        char* ws = lds + kFinishLds + 16;
        if (a.accept_mode == 1 && a.mode == 1) {
            // Review by the rejection rule (the acceptance of the speculative-decoding methods the paper compares
            // with, Section 4.2): draft x at position q, drawn from the small model's nucleus distribution p_S, is kept
            // iff u_acc[q] * p_S(x) < p_L(x); the first refused draft is replaced by a draw from the positive part of
            // p_L - p_S.  Every thread follows the same scalars; the searches and the walk use the whole workgroup.
            const int n = a.T - 1, V = a.vocab;
            int r = n;
            uint32_t KL = 0;
            float massL = 1.f;
            for (int i = 0; i < n; ++i) {
                const int pos = c_ds + i;
                const int x = a.y[pos];
                const float* zl = a.logits + (size_t)(a.row_off + i) * V;
                if (a.top_p < 1.f) nucleus_search(zl, V, rm[i], a.top_p, ws, KL, massL);
                else { KL = 0u; massL = rsum[i]; }
                const float zlx = zl[x];
                const float pl = float_key(zlx) >= KL ? expf(zlx - rm[i]) / massL : 0.f;
                const float4 sd = a.s_draw[pos];  // (max logit, threshold key, nucleus mass) of the small model's row
                const float zsx = a.s_ring[(size_t)i * V + x];
                const float ps = float_key(zsx) >= __float_as_uint(sd.y) ? expf(zsx - sd.x) / sd.z : 0.f;
                if (!(a.u_acc[pos] * ps < pl)) {
                    r = i;
                    break;
                }
            }
            r_given = r;
            const int pos = c_ds + r;
            const float* zl = a.logits + (size_t)(a.row_off + r) * V;
            if (r == n) {
                drawn = nucleus_draw(zl, V, rm[r], a.top_p, a.u[pos], ws);
            } else {  // (KL, massL) are those of row r, the last one searched
                const float4 sd = a.s_draw[pos];
                const float* zs = a.s_ring + (size_t)r * V;
                const uint32_t KS = __float_as_uint(sd.y);
                const float mL = rm[r], iL = 1.f / massL, mS = sd.x, iS = 1.f / sd.z;
                drawn = weighted_walk([&](int v) {
                    const float a_ = zl[v], b_ = zs[v];
                    const float pl = float_key(a_) >= KL ? expf(a_ - mL) * iL : 0.f;
                    const float ps = float_key(b_) >= KS ? expf(b_ - mS) * iS : 0.f;
                    return fmaxf(pl - ps, 0.f);
                }, V, -1.f, a.u[pos], ws);
            }
        } else {
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
            const float* zr = a.logits + (size_t)(a.row_off + row) * a.vocab;
            if (a.accept_mode == 1 && a.mode == 0) {
                // the small model's step under the rejection rule: the review will need the distribution this token was
                // drawn from - keep the row's logits in the slot of its draft index and its (max, threshold, mass)
                uint32_t K;
                float mass;
                nucleus_search(zr, a.vocab, rm[row], a.top_p, ws, K, mass);
                drawn = weighted_walk([&](int i) { const float zi = zr[i]; return float_key(zi) >= K ? expf(zi - rm[row]) : 0.f; },
                                      a.vocab, mass, a.u[pos], ws);
                const int slot = min(max(c_ylen - c_ds, 0), kMaxRows - 1);
                float* dst = a.s_ring + (size_t)slot * a.vocab;
                for (int i = tid; i < a.vocab; i += nthr) dst[i] = zr[i];
                if (tid == 0) a.s_draw[pos] = make_float4(rm[row], __uint_as_float(K), mass, 0.f);
            } else {
                drawn = nucleus_draw(zr, a.vocab, rm[row], a.top_p, a.u[pos], ws);
            }
        }
    }
    // The results go to the control block and, for the caller, to its mirror in pinned host memory: every changed word
    // is written to both from here (the unchanged words of the mirror are the host's own); the pass counter goes last,
    // behind a system-wide fence, so that a host that sees the new count also sees every other word.
    Ctl* hm = a.host_mirror;
    float* nlls = (float*)(ridx + kMaxRows);  // [kMaxRows] (mode 1)
    if (a.mode == 1 && tid < a.T - 1) nlls[tid] = (rm[tid] + logf(rsum[tid])) - a.zt[a.row_off + tid];  // -ln p_L(draft)
    if (a.mode != 3 && tid < a.T) {
        c->res_rowtok[tid] = ridx[tid];
        if (hm) ((volatile int*)hm->res_rowtok)[tid] = ridx[tid];
    }
    __syncthreads();
    if (a.mode == 1 && tid < a.T - 1 && (r_given < 0 || tid <= r_given)) {
        c->res_nll[tid] = nlls[tid];
        if (hm) ((volatile float*)hm->res_nll)[tid] = nlls[tid];
    }
    if (tid == 0) {
        const int w = a.which;
        const int y_len = c_ylen, ds = c_ds, n_max = c_nmax;
        int n_ylen = y_len, n_ds = ds, n_len0 = c_len0, n_lenw = c_lenw;
        int res_tok = 0, res_flag = 0, res_r = 0, res_n = 0;
        float res_pmax = 0.f;
        if (a.mode == 3) {
            n_lenw = c_lenw + a.rows_consumed;
        } else if (a.mode == 0 || a.mode == 2) {
            const int tok = drawn >= 0 ? drawn : ridx[a.T - 1];
            const float pmax = 1.f / rsum[a.T - 1];
            const bool low = (a.mode == 0) && (pmax < c_afb);
            const bool forced = (a.mode == 0) && n_max > 0 && (y_len - ds) >= n_max;
            const bool fb = low || forced;
            n_lenw = c_lenw + a.rows_consumed;
            if (!fb && y_len < a.y_cap) {
                a.y[y_len] = tok;
                n_ylen = y_len + 1;
                if (a.mode == 2) n_ds = y_len + 1;
            }
            res_tok = tok;
            res_flag = (fb ? 1 : 0) | ((forced && !low) ? 2 : 0);
            res_pmax = pmax;
        } else if (a.mode == 1) {  // review of n = T - 1 drafts
            const int n = a.T - 1;
            const float alpha = c_arb;
            int r = n;
            if (r_given >= 0) {
                r = r_given;  // (the rejection rule decided above)
            } else {
                for (int i = 0; i < n; ++i)
                    if (nlls[i] > alpha) {
                        r = i;
                        break;
                    }
            }
            const int tok = drawn >= 0 ? drawn : ridx[r];
            a.y[ds + r] = tok;
            n_ylen = ds + r + 1;
            n_lenw = ds + r;            // (w == 1)
            n_len0 = min(c_len0, ds + r);
            n_ds = ds + r + 1;
            res_r = r;
            res_n = n;
            res_tok = tok;
            res_pmax = 1.f / rsum[r];
        }
        if (a.mode != 4) {
            const int l0 = w == 0 ? n_lenw : n_len0, l1 = w == 1 ? n_lenw : c->len[1];
            c->y_len = n_ylen; c->draft_start = n_ds; c->len[0] = l0; c->len[1] = l1;
            c->res_tok = res_tok; c->res_flag = res_flag; c->res_r = res_r; c->res_n = res_n; c->res_pmax = res_pmax;
            if (hm) {
                volatile Ctl* v = hm;
                v->y_len = n_ylen; v->draft_start = n_ds; v->len[0] = l0; v->len[1] = l1;
                v->res_tok = res_tok; v->res_flag = res_flag; v->res_r = res_r; v->res_n = res_n; v->res_pmax = res_pmax;
            }
        }
    }
    if (hm) {
        static_assert(offsetof(Ctl, seq) == sizeof(Ctl) - 4, "seq must be the last word of the control block");
        __threadfence_system();
        __syncthreads();
        if (tid == 0) {
            const int sq = c_seq + 1;
            c->seq = sq;
            ((volatile Ctl*)hm)->seq = sq;
        }
    }
}

__global__ __launch_bounds__(256) void finish_kernel(const FinishArgs a) {
    __shared__ __attribute__((aligned(16))) char lds[kFinishLds];
    finish_body<false>(a, lds);
}

// Reviews of several rows: sixteen waves, so that the rows' partial statistics are merged side by side (a wave takes
// rows w, w + 16, ...: one trip to memory per row it has).
__global__ __launch_bounds__(1024) void finish_wide_kernel(const FinishArgs a) {
    __shared__ __attribute__((aligned(16))) char lds[kFinishLds];
    finish_body<false>(a, lds);
}

__global__ __launch_bounds__(1024) void finish_sample_kernel(const FinishArgs a) {
    __shared__ __attribute__((aligned(16))) char lds[kFinishLds + 16 + kDrawLds];
    finish_body<true>(a, lds);
}


// =====================================================================================
// Nucleus draw spread over the chip (sampling variant with the threshold rule of the review).
//
// The single-workgroup draw above sweeps a row of logits eight times on one compute unit (80 us at 32 128 ids, 650 us
// at 250 112).  Here the row is cut into slices of kDrawSliceIds ids, one workgroup each, and every probability mass
// is an INTEGER: exp(z - max) in units of 2^-40, truncated.  Integer sums do not depend on the order of their terms,
// so masses can be added with atomics and the result is still the same on every run; and the nucleus mass found by the
// threshold search equals the sum of the members' masses of the walk exactly, so the walk always ends inside the nucleus.
//
//   draw_select_kernel   (1 workgroup)  merges the LM-head partials, applies the rollback test to find the row the
//                        token comes from, leaves (row, position, max) and the merged statistics in the workspace,
//                        clears the histograms
//   draw_sweep_kernel<L> (slices)       L = 0..3: mass per value of key byte 3-L among the ids whose higher key bytes
//                        equal the threshold's (every workgroup re-derives those bytes from the earlier histograms)
//   draw_mass_kernel     (slices)       threshold key and nucleus mass complete; members' mass per slice
//   finish_draw_kernel   (1 workgroup)  floor(u * mass) -> slice -> id by two integer prefix sums; then the policy and
//                        the commit of finish_body with that token
// =====================================================================================
typedef unsigned long long u64;

__device__ __forceinline__ u64 mass_units(float z, float m) { return (u64)(expf(z - m) * 1099511627776.f); }  // 2^40

// Sums over the 256 threads of a workgroup: inside each wavefront by lane shifts (no barrier), then the four wave totals
// through LDS (buf: 4 words).  Both end with a barrier, so buf may be reused at once.
__device__ __forceinline__ u64 suffix_sum_256(u64 v, u64* buf) {  // sum over the threads at and above this one
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const u64 t = __shfl_down(v, off, 64);
        if (lane + off < 64) v += t;
    }
    if (lane == 0) buf[wave] = v;
    __syncthreads();
    u64 add = 0;
#pragma unroll
    for (int w = 1; w < 4; ++w)
        if (w > wave) add += buf[w];
    __syncthreads();
    return v + add;
}
__device__ __forceinline__ u64 prefix_excl_256(u64 v, u64* buf) {  // sum over the threads below this one
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    u64 acc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const u64 t = __shfl_up(acc, off, 64);
        if (lane >= off) acc += t;
    }
    if (lane == 63) buf[wave] = acc;
    __syncthreads();
    u64 add = 0;
#pragma unroll
    for (int w = 0; w < 3; ++w)
        if (w < wave) add += buf[w];
    __syncthreads();
    return acc + add - v;
}

// The threshold's key bytes decided by histograms 0..LEVELS-1 (thread j holds bin j of each), the mass of the keys
// strictly above that prefix's range, and the target top_p * total.  With S_l[j] the mass of bins j.. of level l, the byte
// of level l is the largest j with above + S_l[j] >= target (0 if none); `in_play` returns the mass of that bin onward.
// lds: 256 u64 + 8 u64.  All threads return the same values.
template <int LEVELS>
__device__ __forceinline__ void threshold_prefix(const DrawWs* ws, float top_p, u64* lds, uint32_t& K, u64& above, u64& at_or_above) {
    const int tid = threadIdx.x;
    u64 h[LEVELS > 0 ? LEVELS : 1];
#pragma unroll
    for (int l = 0; l < LEVELS; ++l) h[l] = ws->hist[l][tid];
    u64* sc = lds + 256;
    K = 0;
    above = 0;
    at_or_above = 0;
    u64 target = 0;
#pragma unroll
    for (int l = 0; l < LEVELS; ++l) {
        const u64 S = suffix_sum_256(h[l], lds);       // mass of bins tid..255
        if (l == 0) {
            if (tid == 0) sc[0] = (u64)ceil((double)top_p * (double)S);
            __syncthreads();
            target = sc[0];
        }
        const u64 Snext = S - h[l];                    // mass of bins tid+1..255
        const bool here = above + S >= target || tid == 0;
        const bool next = tid < 255 && above + Snext >= target;
        if (here && !next) {                           // exactly one thread
            sc[1] = (u64)tid;
            sc[2] = above + Snext;
            sc[3] = above + S;
        }
        __syncthreads();
        K |= (uint32_t)sc[1] << (24 - 8 * l);
        above = sc[2];
        at_or_above = sc[3];
        __syncthreads();
    }
}

__global__ __launch_bounds__(1024) void draw_select_kernel(const FinishArgs a) {
    __shared__ __attribute__((aligned(16))) char lds[kFinishLds];
    float* rm = (float*)lds;
    float* rsum = rm + kMaxRows;
    int* ridx = (int*)(rsum + kMaxRows);
    const int tid = threadIdx.x;
    const Ctl* c = a.ctl;
    const int c_ylen = c->y_len, c_ds = c->draft_start;
    const float c_arb = c->alpha_rb;
    DrawWs* ws = a.dws;
    u64* hist = &ws->hist[0][0];
    for (int i = tid; i < 4 * 256; i += blockDim.x) hist[i] = 0ull;
    merge_partials(a, rm, rsum, ridx);
    if (tid < a.T) {
        StatPart sp;
        sp.m = rm[tid]; sp.s = rsum[tid]; sp.idx = ridx[tid]; sp.pad = 0;
        ws->merged[a.row_off + tid] = sp;
    }
    if (tid == 0) {
        int row = a.T - 1, pos = c_ylen;
        if (a.mode == 1) {  // review: the first draft whose cross-entropy exceeds the threshold (Section 3.4), else the row after the last
            const int n = a.T - 1;
            row = n;
            for (int i = 0; i < n; ++i)
                if ((rm[i] + logf(rsum[i])) - a.zt[a.row_off + i] > c_arb) {
                    row = i;
                    break;
                }
            pos = c_ds + row;
        }
        ws->row = row;
        ws->pos = pos;
        ws->m = rm[row];
    }
}

template <int L>
__global__ __launch_bounds__(256) void draw_sweep_kernel(const FinishArgs a) {
    __shared__ u64 lds[256 + 8];
    __shared__ u64 bins[256];
    const int tid = threadIdx.x;
    const DrawWs* ws = a.dws;
    const int row = ws->row;
    const float m = ws->m;
    const float* z = a.logits + (size_t)(a.row_off + row) * a.vocab;
    constexpr int PER = kDrawSliceIds / 256;
    const int i0 = (int)blockIdx.x * kDrawSliceIds + tid;
    float zi[PER];
#pragma unroll
    for (int c = 0; c < PER; ++c) zi[c] = z[min(i0 + c * 256, a.vocab - 1)];
    bins[tid] = 0ull;
    uint32_t K = 0;
    u64 above, at;
    threshold_prefix<L>(ws, a.top_p, lds, K, above, at);  // (barriers inside; L == 0: none, hence the one below)
    __syncthreads();
    constexpr int shift = 24 - 8 * L;
#pragma unroll
    for (int c = 0; c < PER; ++c) {
        const uint32_t k = float_key(zi[c]);
        bool mine = i0 + c * 256 < a.vocab;
        if constexpr (L > 0) mine = mine && ((k ^ K) >> (shift + 8)) == 0u;  // the higher key bytes are the threshold's
        if (mine) {
            const u64 e = mass_units(zi[c], m);
            if (e) atomicAdd(&bins[(k >> shift) & 255u], e);
        }
    }
    __syncthreads();
    const u64 mine = bins[tid];
    if (mine) atomicAdd(&a.dws->hist[L][tid], mine);
}

__global__ __launch_bounds__(256) void draw_mass_kernel(const FinishArgs a) {
    __shared__ u64 lds[256 + 8];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    DrawWs* ws = a.dws;
    const int row = ws->row;
    const float m = ws->m;
    const float* z = a.logits + (size_t)(a.row_off + row) * a.vocab;
    constexpr int PER = kDrawSliceIds / 256;
    const int i0 = (int)blockIdx.x * kDrawSliceIds + tid;
    float zi[PER];
#pragma unroll
    for (int c = 0; c < PER; ++c) zi[c] = z[min(i0 + c * 256, a.vocab - 1)];
    uint32_t K;
    u64 above, at;
    threshold_prefix<4>(ws, a.top_p, lds, K, above, at);
    u64 mine = 0;
#pragma unroll
    for (int c = 0; c < PER; ++c)
        if (i0 + c * 256 < a.vocab && float_key(zi[c]) >= K) mine += mass_units(zi[c], m);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o, 64);
    if (lane == 0) lds[wave] = mine;
    __syncthreads();
    if (tid == 0) {
        ws->slice[blockIdx.x] = lds[0] + lds[1] + lds[2] + lds[3];
        if (blockIdx.x == 0) {
            ws->key = K;
            ws->mass = at;  // every key >= K: the mass above the last byte's bin plus that bin's
        }
    }
}

__global__ __launch_bounds__(256) void finish_draw_kernel(const FinishArgs a, const int nslices) {
    __shared__ __attribute__((aligned(16))) char lds[kFinishLds];
    __shared__ u64 buf[256];
    __shared__ u64 sc[4];
    const int tid = threadIdx.x;
    const DrawWs* ws = a.dws;
    const int row = ws->row, pos = ws->pos;
    const float m = ws->m;
    const uint32_t K = ws->key;
    const u64 mass = ws->mass;
    const float u = a.u[pos];
    // target: the first member (ids increasing) whose running mass exceeds u * mass, i.e. exceeds t = floor(u * mass)
    const u64 t = (u64)((double)u * (double)mass);
    // ---- slice ----
    constexpr int SPT = kDrawMaxSlices / 256;  // slices per thread, consecutive
    u64 sm[SPT], mine = 0;
#pragma unroll
    for (int k = 0; k < SPT; ++k) {
        const int sl = tid * SPT + k;
        sm[k] = sl < nslices ? ws->slice[sl] : 0ull;
        mine += sm[k];
    }
    const u64 before = prefix_excl_256(mine, buf);
    if (tid == 0) { sc[0] = 0; sc[1] = 0; }
    __syncthreads();
    if (before <= t && t < before + mine) {  // exactly one thread (the masses add up to `mass` > t exactly)
        u64 run = before;
        int k = 0;
        for (; k < SPT - 1; ++k) {
            if (t < run + sm[k]) break;
            run += sm[k];
        }
        sc[0] = (u64)(tid * SPT + k);
        sc[1] = run;
    }
    __syncthreads();
    const int sl = (int)sc[0];
    const u64 rem = t - sc[1];  // mass to pass inside the slice
    __syncthreads();
    // ---- id inside the slice: thread j owns ids 4j .. 4j+3 of it ----
    const float* z = a.logits + (size_t)(a.row_off + row) * a.vocab;
    constexpr int PER = kDrawSliceIds / 256;
    const int i0 = sl * kDrawSliceIds + tid * PER;
    u64 e[PER], tot = 0;
#pragma unroll
    for (int c = 0; c < PER; ++c) {
        const float zi = z[min(i0 + c, a.vocab - 1)];
        e[c] = (i0 + c < a.vocab && float_key(zi) >= K) ? mass_units(zi, m) : 0ull;
        tot += e[c];
    }
    const u64 bef = prefix_excl_256(tot, buf);
    if (tid == 0) sc[2] = (u64)(uint32_t)ws->merged[a.row_off + row].idx;  // (never used: rem < the slice's mass)
    __syncthreads();
    if (bef <= rem && rem < bef + tot) {
        u64 run = bef;
        int c = 0;
        for (; c < PER - 1; ++c) {
            run += e[c];
            if (run > rem) break;
        }
        sc[2] = (u64)(i0 + c);
    }
    __syncthreads();
    finish_body<false>(a, lds, (int)sc[2]);
}

hipError_t launch_finish_draw(const FinishArgs& a, hipStream_t st) {
    if (!(a.top_p > 0.f) || a.mode > 2 || a.accept_mode != 0 || !a.logits || !a.u || !a.dws || a.vocab < 1 || a.T < 1 || a.T > kMaxRows)
        return hipErrorInvalidValue;
    const int ns = (a.vocab + kDrawSliceIds - 1) / kDrawSliceIds;
    if (ns > kDrawMaxSlices) return hipErrorInvalidValue;
    hipLaunchKernelGGL(draw_select_kernel, dim3(1), dim3(a.T > 4 || a.nparts > 1024 ? 1024 : 256), 0, st, a);
    hipLaunchKernelGGL(draw_sweep_kernel<0>, dim3(ns), dim3(256), 0, st, a);
    hipLaunchKernelGGL(draw_sweep_kernel<1>, dim3(ns), dim3(256), 0, st, a);
    hipLaunchKernelGGL(draw_sweep_kernel<2>, dim3(ns), dim3(256), 0, st, a);
    hipLaunchKernelGGL(draw_sweep_kernel<3>, dim3(ns), dim3(256), 0, st, a);
    hipLaunchKernelGGL(draw_mass_kernel, dim3(ns), dim3(256), 0, st, a);
    FinishArgs f = a;  // the commit merges one "partial" per row: the statistics draw_select_kernel left
    f.part = a.dws->merged;  // (address arithmetic only: dws is a device pointer)
    f.nparts = 1;
    hipLaunchKernelGGL(finish_draw_kernel, dim3(1), dim3(256), 0, st, f, ns);
    return hipGetLastError();
}

hipError_t launch_finish(const FinishArgs& a, hipStream_t st) {
    if (a.top_p > 0.f && a.mode <= 2) {
        if (!a.logits || !a.u || a.vocab < 1) return hipErrorInvalidValue;
        if (a.accept_mode == 1 && (!a.u_acc || !a.s_ring || !a.s_draw)) return hipErrorInvalidValue;
        hipLaunchKernelGGL(finish_sample_kernel, dim3(1), dim3(1024), 0, st, a);
        return hipGetLastError();
    }
    if (a.mode != 3 && (a.T > 4 || a.nparts > 1024)) hipLaunchKernelGGL(finish_wide_kernel, dim3(1), dim3(1024), 0, st, a);
    else hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace bild
