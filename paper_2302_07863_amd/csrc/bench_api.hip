// Measurement, probe and host-logic entry points (include/bild_bench.h): timing of passes and of the
// weight-streaming GEMM, the plain kernels hardware counters are scaled against, and the host-side
// layout / launch-shape logic exposed for CPU tests.  Nothing here takes part in decoding.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <vector>

#include "bild_bench.h"
#include "bild_state.h"

using namespace bild;

namespace bild {

// Plain copy of known size: the reference against which hardware byte counters are scaled.
__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// A kernel that does nothing on one workgroup per CU: what a dependent launch costs by itself.
__global__ __launch_bounds__(256) void probe_empty_kernel() {}

static hipError_t launch_probe_empty(hipStream_t st) {
    hipLaunchKernelGGL(probe_empty_kernel, dim3(256), dim3(256), 0, st);
    return hipGetLastError();
}

// Every workgroup (8 waves) streams a private contiguous region, 16 tiles of 1 KiB per wave in flight: how fast
// ONE compute unit can pull from HBM, and how the total grows with the number of workgroups.
__global__ __launch_bounds__(512) void probe_stream_kernel(const uint4* __restrict__ p, size_t tiles_per_wg, uint4* sink) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const uint4* base = p + (size_t)blockIdx.x * tiles_per_wg * 64 + lane;
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (size_t t = wave; t < tiles_per_wg; t += 8 * 16) {
        uint4 v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = base[min(t + (size_t)u * 8, tiles_per_wg - 1) * 64];
#pragma unroll
        for (int u = 0; u < 16; ++u) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
    }
    if (acc.x == 0x12345678u && acc.y == 0x9abcdefu) sink[0] = acc;  // keeps the loads alive; never true for zeroed memory
}

static hipError_t launch_probe_stream(const void* src, size_t kib_per_group, int groups, void* sink, hipStream_t st) {
    hipLaunchKernelGGL(probe_stream_kernel, dim3(groups), dim3(512), 0, st, (const uint4*)src, kib_per_group, (uint4*)sink);
    return hipGetLastError();
}

static hipError_t launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t st) {
    hipLaunchKernelGGL(probe_copy_kernel, dim3(4096), dim3(256), 0, st, (const uint4*)src, (uint4*)dst, bytes / 16);
    return hipGetLastError();
}


}  // namespace bild

extern "C" int bild_bench_pass(bild_state* s, int which, int rows, int reps, float* ms_per_pass) {
    if (!s || !ms_per_pass || which < 1 || which > 2 || rows < 1 || rows > kMaxRows || reps < 1) return BILD_EINVAL;
    if (!s->encoded) return BILD_ESTATE;
    const int w = which - 1;
    if (s->y_len - s->len[w] < rows) return BILD_ESTATE;
    int rc = catch_up(s, w, s->y_len - rows);  // the timed passes cover exactly the last `rows` tokens
    if (rc) return rc;
    hipEvent_t e0, e1;
    HIPC(hipEventCreate(&e0));
    HIPC(hipEventCreate(&e1));
    rc = run_pass(s, w, rows, rows, 4);  // warm-up (and graph capture)
    if (rc == BILD_OK && hipEventRecord(e0, s->stream) != hipSuccess) rc = BILD_EHIP;
    for (int i = 0; i < reps && rc == BILD_OK; ++i) rc = run_pass(s, w, rows, rows, 4);
    if (rc == BILD_OK && hipEventRecord(e1, s->stream) != hipSuccess) rc = BILD_EHIP;
    if (rc == BILD_OK && hipEventSynchronize(e1) != hipSuccess) rc = BILD_EHIP;
    float ms = 0.f;
    if (rc == BILD_OK && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = BILD_EHIP;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc) return rc;
    *ms_per_pass = ms / (float)reps;
    return BILD_OK;
}

extern "C" int bild_bench_gemm(bild_state* s, int which, int rows, int reps, float* ms_per_pass, int64_t* launches,
                               int64_t* bytes) {
    if (!s || !ms_per_pass || !launches || !bytes || which < 1 || which > 2 || rows < 1 || rows > kMaxRows || reps < 1)
        return BILD_EINVAL;
    if (!s->encoded) return BILD_ESTATE;
    const int w = which - 1;
    if (s->y_len - s->len[w] < rows) return BILD_ESTATE;
    int rc = catch_up(s, w, s->y_len - rows);
    if (rc) return rc;
    hipEvent_t e0, e1;
    HIPC(hipEventCreate(&e0));
    HIPC(hipEventCreate(&e1));
    s->gemm_only = true;
    s->gemm_count = s->gemm_bytes = 0;
    const bool graphs = s->use_graphs;
    s->use_graphs = false;
    rc = decoder_pass(s, w, rows, rows, 4, key_bucket(s->len[w] + rows));  // count the launches of one pass
    s->use_graphs = graphs;
    *launches = s->gemm_count;
    *bytes = s->gemm_bytes;
    if (rc == BILD_OK) rc = run_pass(s, w, rows, rows, 4);  // warm-up / capture
    if (rc == BILD_OK && hipEventRecord(e0, s->stream) != hipSuccess) rc = BILD_EHIP;
    for (int i = 0; i < reps && rc == BILD_OK; ++i) rc = run_pass(s, w, rows, rows, 4);
    if (rc == BILD_OK && hipEventRecord(e1, s->stream) != hipSuccess) rc = BILD_EHIP;
    if (rc == BILD_OK && hipEventSynchronize(e1) != hipSuccess) rc = BILD_EHIP;
    s->gemm_only = false;
    float ms = 0.f;
    if (rc == BILD_OK && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = BILD_EHIP;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc) return rc;
    *ms_per_pass = ms / (float)reps;
    return BILD_OK;
}

extern "C" int bild_pass_stages(bild_state* s, int32_t* stages) {
    if (!s || !stages) return BILD_EINVAL;
    *stages = s->stage_count;
    return BILD_OK;
}

extern "C" int bild_gemm_tally(bild_state* s, int64_t* launches, int64_t* bytes, int reset) {
    if (!s || !launches || !bytes) return BILD_EINVAL;
    *launches = s->gemm_count;
    *bytes = s->gemm_bytes;
    if (reset) s->gemm_count = s->gemm_bytes = 0;
    return BILD_OK;
}

extern "C" int bild_probe_launch(bild_state* s, int reps, float* us_per_launch) {
    if (!s || reps < 1 || !us_per_launch) return BILD_EINVAL;
    hipEvent_t e0, e1;
    HIPC(hipEventCreate(&e0));
    HIPC(hipEventCreate(&e1));
    int rc = BILD_OK;
    for (int i = 0; i < 16 && rc == BILD_OK; ++i)
        if (launch_probe_empty(s->stream) != hipSuccess) rc = BILD_EHIP;
    if (rc == BILD_OK && hipEventRecord(e0, s->stream) != hipSuccess) rc = BILD_EHIP;
    for (int i = 0; i < reps && rc == BILD_OK; ++i)
        if (launch_probe_empty(s->stream) != hipSuccess) rc = BILD_EHIP;
    if (rc == BILD_OK && hipEventRecord(e1, s->stream) != hipSuccess) rc = BILD_EHIP;
    if (rc == BILD_OK && hipEventSynchronize(e1) != hipSuccess) rc = BILD_EHIP;
    float ms = 0.f;
    if (rc == BILD_OK && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = BILD_EHIP;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc == BILD_OK) *us_per_launch = ms * 1e3f / (float)reps;
    return rc;
}

extern "C" int bild_probe_stream(bild_state* s, int groups, int kib_per_group, int reps, float* us_per_launch) {
    if (!s || !us_per_launch || groups < 1 || groups > 4096 || kib_per_group < 1 || kib_per_group > (1 << 16) || reps < 1 || reps > 64)
        return BILD_EINVAL;
    // every launch reads a region no earlier launch touched, so nothing comes from a cache
    const size_t per_launch = (size_t)groups * kib_per_group * 1024;
    if (per_launch * (size_t)(reps + 1) > ((size_t)16 << 30)) return BILD_EINVAL;
    void *buf = nullptr, *sink = nullptr;
    if (hipMalloc(&buf, per_launch * (reps + 1)) != hipSuccess) return BILD_ENOMEM;
    if (hipMalloc(&sink, 64) != hipSuccess) {
        (void)hipFree(buf);
        return BILD_ENOMEM;
    }
    int rc = BILD_OK;
    if (hipMemsetAsync(buf, 0, per_launch * (reps + 1), s->stream) != hipSuccess) rc = BILD_EHIP;
    if (rc == BILD_OK && launch_probe_stream(buf, (size_t)kib_per_group, groups, sink, s->stream) != hipSuccess) rc = BILD_EHIP;  // warm-up
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (rc == BILD_OK && (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)) rc = BILD_EHIP;
    float total_ms = 0.f;
    // one bracket around all launches: launches on one stream run one after the other, so the mean holds the same
    // launch-to-launch gap a stage of a pass pays, and not the cost of the events
    if (rc == BILD_OK && hipEventRecord(e0, s->stream) != hipSuccess) rc = BILD_EHIP;
    for (int i = 0; i < reps && rc == BILD_OK; ++i) {
        const char* region = (const char*)buf + per_launch * (size_t)(i + 1);
        if (launch_probe_stream(region, (size_t)kib_per_group, groups, sink, s->stream) != hipSuccess) rc = BILD_EHIP;
    }
    if (rc == BILD_OK && (hipEventRecord(e1, s->stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                          hipEventElapsedTime(&total_ms, e0, e1) != hipSuccess))
        rc = BILD_EHIP;
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipStreamSynchronize(s->stream);
    (void)hipFree(buf);
    (void)hipFree(sink);
    if (rc == BILD_OK) *us_per_launch = total_ms * 1e3f / (float)reps;
    return rc;
}

extern "C" int bild_probe_copy(bild_state* s, int64_t bytes, int reps) {
    if (!s || bytes < 16 || bytes % 16 || reps < 1) return BILD_EINVAL;
    void *a = nullptr, *b = nullptr;
    if (hipMalloc(&a, (size_t)bytes) != hipSuccess) return BILD_ENOMEM;
    if (hipMalloc(&b, (size_t)bytes) != hipSuccess) {
        (void)hipFree(a);
        return BILD_ENOMEM;
    }
    int rc = BILD_OK;
    if (hipMemsetAsync(a, 1, (size_t)bytes, s->stream) != hipSuccess) rc = BILD_EHIP;
    for (int i = 0; i < reps && rc == BILD_OK; ++i)
        if (launch_probe_copy(a, b, (size_t)bytes, s->stream) != hipSuccess) rc = BILD_EHIP;
    if (hipStreamSynchronize(s->stream) != hipSuccess) rc = BILD_EHIP;
    (void)hipFree(a);
    (void)hipFree(b);
    return rc;
}

extern "C" int bild_profile_begin(bild_state* s, int max_records) {
    if (!s || max_records < 1 || max_records > (1 << 20)) return BILD_EINVAL;
    if (s->prof_on) return BILD_ESTATE;
    while ((int)s->prof_ev.size() < 2 * max_records) {
        hipEvent_t e;
        HIPC(hipEventCreate(&e));
        s->prof_ev.push_back(e);
    }
    s->prof_cap = max_records;
    s->prof_used = 0;
    s->prof_dropped = 0;
    s->prof_rec.clear();
    s->prof_on = true;
    return BILD_OK;
}

extern "C" int bild_profile_end(bild_state* s, bild_profile* out) {
    if (!s || !out) return BILD_EINVAL;
    if (!s->prof_on) return BILD_ESTATE;
    s->prof_on = false;
    HIPC(hipStreamSynchronize(s->stream));
    std::memset(out, 0, sizeof(*out));
    for (int i = 0; i < s->prof_used; ++i) {
        float ms = 0.f;
        HIPC(hipEventElapsedTime(&ms, s->prof_ev[2 * i], s->prof_ev[2 * i + 1]));
        const auto& r = s->prof_rec[i];
        out->launches[r.model][r.cls] += 1;
        out->bytes[r.model][r.cls] += r.bytes;
        out->ms[r.model][r.cls] += ms;
    }
    out->dropped = s->prof_dropped;
    return BILD_OK;
}

extern "C" int64_t bild_pass_bytes(const bild_state* s, int which, int t_cache, int rows) {
    if (!s || which < 1 || which > 2) return BILD_EINVAL;
    const bild_model* m = s->ms[which - 1].m;
    const bild_model_config& c = m->cfg;
    const int64_t d = c.d_model, I = m->inner(), F = c.d_ff, B = m->esz();
    // an early-exit pair's large pass runs the layers above the trunk only
    const int64_t L = c.n_dec_layers - (which == 2 ? s->pair->trunk_layers : 0);
    const int64_t attn = 4 * d * I * (c.cross_attn ? 2 : 1);
    const int64_t ffn = (m->gated() ? 3 : 2) * d * F;
    int64_t elems = L * (attn + ffn) + (int64_t)c.vocab * d + L * 2 * I * (int64_t)(t_cache + rows);
    if (c.cross_attn) elems += L * 2 * I * (int64_t)s->n_src;
    return elems * B;
}

extern "C" int64_t bild_debug_tiled_bytes(int n, int k, int dtype) {
    if (n < 1 || k < 32 || k % 32 || dtype < 0 || dtype > 1) return BILD_EINVAL;
    return (int64_t)tiled_bytes(n, k, dtype);
}

extern "C" int bild_debug_tile_matrix(const float* src, int src_is_k_by_n, int n, int k, int dtype, void* dst) {
    if (!src || !dst || n < 1 || k < 32 || k % 32 || dtype < 0 || dtype > 1) return BILD_EINVAL;
    tile_matrix(src, src_is_k_by_n != 0, n, k, dtype, dst);
    return BILD_OK;
}

extern "C" int bild_debug_gemm_shape(int n, int k, int rows, int gated, int lm_head, int dtype, int32_t out[8]) {
    if (!out || n < 1 || k < 32 || k % 32 || rows < 1 || dtype < 0 || dtype > 1) return BILD_EINVAL;
    if (lm_head && rows > kMaxRows) return BILD_EINVAL;
    GemmArgs g;
    std::memset((void*)&g, 0, sizeof(g));
    const int kt = dtype ? 32 : 16;
    g.W.n = gated ? 2 * n : n;  // gate and linear branch interleaved by tile
    g.W.k = k;
    g.W.tn = (g.W.n + 15) / 16;
    g.W.tk = k / kt;
    g.T = rows;
    g.epi = lm_head ? EPI_LMHEAD : (gated ? EPI_ACT : EPI_STORE);
    g.act = gated ? BILD_ACT_SWIGLU : BILD_ACT_RELU;
    gemm_pick_shape(g, dtype);
    out[0] = g.wk;
    out[1] = g.nwv;
    out[2] = g.rw;
    out[3] = g.kc;
    out[4] = (int32_t)gemm_num_blocks(g);
    out[5] = rows >= kDenseMinRows ? (rows + kDenseRows - 1) / kDenseRows : (rows + kMaxRows - 1) / kMaxRows;
    out[6] = (int32_t)gemm_lds_bytes(g, dtype);
    out[7] = 160 * 1024;
    return BILD_OK;
}

extern "C" int bild_debug_attn_shape(int heads, int d_head, int rows, int nkeys, int max_splits, int dtype, int32_t out[4]) {
    if (!out || heads < 1 || d_head < 8 || d_head > 128 || rows < 1 || nkeys < 1 || max_splits < 1 || dtype < 0 || dtype > 1)
        return BILD_EINVAL;
    bool defer = false;
    const int sp = rows > kMaxRows ? 1 : pick_splits_raw(d_head, dtype ? 2 : 4, max_splits, nkeys, heads, rows, &defer);
    const int nw = pick_attn_waves(dtype, d_head, std::min(rows, kMaxRows), nkeys, sp);
    out[0] = sp;
    out[1] = (sp > 1 && defer) ? 1 : 0;
    out[2] = nw;
    out[3] = (int32_t)attn_lds_bytes(dtype, d_head, std::min(rows, kMaxRows), nw);
    return BILD_OK;
}

