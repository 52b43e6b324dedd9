// bild_head_stats / bild_head_stats_static: the final norm + LM head + softmax statistics of the decoding path
// (the fused vocabulary sweep of a decoder pass) as a call of its own on hidden rows the caller already holds
// on the device.  Both entry points run the same kernels; they differ only in where the scratch buffer lives
// (per-workgroup partial statistics, the logits of the targets, one length word):
//   bild_head_stats         allocates it with hipMalloc for the call and frees it before returning;
//   bild_head_stats_static  uses a file-scope device array, so the call allocates nothing at all.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>

#include "bild_state.h"

using namespace bild;

namespace {

// Scratch layout (bytes): [0, 256) one int (number of target slots); [256, 512) logits of the targets, one float per
// row; [512, ...) partial statistics, StatPart[workgroups][kMaxRows].
constexpr size_t kHdrBytes = 512;
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;  // 4 MiB
constexpr int kStaticMaxParts = (int)((kStaticScratchBytes - kHdrBytes) / (sizeof(StatPart) * kMaxRows));

// One copy per GPU the library runs on, kept until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress: the device address of the array is looked up once per device (scratch_of_device) and that
// pointer is what kernels and every other call receive.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};

int scratch_of_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return BILD_EHIP;
    void* p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return BILD_EHIP;
        __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);
    }
    *out = p;
    return BILD_OK;
}

// Writes the number of target slots (rows + 1, or 0 for "no targets") and clears the target logits.
__global__ __launch_bounds__(64) void head_stats_setup_kernel(int* nslots, float* zt, int value) {
    if (threadIdx.x == 0) *nslots = value;
    if (threadIdx.x < kMaxRows) zt[threadIdx.x] = __builtin_nanf("");
}

struct MergeArgs {
    const StatPart* part;
    int nparts;
    const float* zt;
    int rows;
    int has_targets;
    bild_row_stats* out;
};

// One wave per row: merges the per-workgroup partial statistics in a fixed order and writes the row's result.
__global__ __launch_bounds__(256) void head_stats_merge_kernel(const MergeArgs a) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwv = blockDim.x >> 6;
    for (int t = wave; t < a.rows; t += nwv) {
        float m = -INFINITY, s = 0.f;
        int idx = 0x7FFFFFFF;
        for (int p = lane; p < a.nparts; p += 64) {
            const StatPart sp = a.part[(size_t)p * kMaxRows + t];
            const float mn = fmaxf(m, sp.m);
            const float sa = (m == -INFINITY) ? 0.f : s * expf(m - mn);
            const float sb = (sp.m == -INFINITY) ? 0.f : sp.s * expf(sp.m - mn);
            idx = (m > sp.m || (m == sp.m && idx < sp.idx)) ? idx : sp.idx;
            m = mn;
            s = sa + sb;
        }
        for (int o = 32; o > 0; o >>= 1) {
            const float m2 = __shfl_xor(m, o, 64), s2 = __shfl_xor(s, o, 64);
            const int i2 = __shfl_xor(idx, o, 64);
            const float mn = fmaxf(m, m2);
            const float sa = (m == -INFINITY) ? 0.f : s * expf(m - mn);
            const float sb = (m2 == -INFINITY) ? 0.f : s2 * expf(m2 - mn);
            idx = (m > m2 || (m == m2 && idx < i2)) ? idx : i2;
            m = mn;
            s = sa + sb;
        }
        if (lane == 0) {
            bild_row_stats r;
            r.zmax = m;
            r.lse = m + logf(s);
            r.argmax = idx;
            r.z_target = a.has_targets ? a.zt[t] : __builtin_nanf("");
            a.out[t] = r;
        }
    }
}

// The launch shape of the head for `rows` rows; *nparts receives the number of workgroups (partials per row).
GemmArgs head_gemm(const bild_model* m, const float* x, int rows, const int32_t* targets, void* scr) {
    GemmArgs g;
    std::memset((void*)&g, 0, sizeof(g));
    const bild_model_config& c = m->cfg;
    g.W = m->head;
    g.x = x;
    g.ldx = c.d_model;
    g.T = rows;
    g.gain = m->dec_final;
    g.eps = c.norm_eps;
    g.d_head = c.d_head;
    g.i_dim = m->inner();
    g.rope_base = c.rope_base;
    g.act = c.act;
    g.vocab = c.vocab;
    g.epi = EPI_LMHEAD;
    g.scale = c.logit_scale;
    // the kernel takes the target of row t from y[t + 1] while t + 1 < *ylen_ptr: y is the caller's array moved down
    // by one slot, and the slot count is rows + 1 (0 without targets, so that y is never read)
    g.y = targets ? targets - 1 : (const int*)scr;
    g.ylen_ptr = (const int*)scr;
    g.zt = (float*)((char*)scr + 256);
    g.part = (StatPart*)((char*)scr + kHdrBytes);
    gemm_pick_shape(g, c.dtype);
    return g;
}

int head_stats_run(const bild_model* m, const float* x, int rows, const int32_t* targets, bild_row_stats* out,
                   hipStream_t st, void* scr, const GemmArgs& g) {
    hipLaunchKernelGGL(head_stats_setup_kernel, dim3(1), dim3(64), 0, st, (int*)scr, (float*)((char*)scr + 256),
                       targets ? rows + 1 : 0);
    HIPC(hipGetLastError());
    HIPC(launch_gemm(g, m->cfg.dtype, st));
    MergeArgs ma;
    ma.part = g.part;
    ma.nparts = (int)gemm_num_blocks(g);
    ma.zt = g.zt;
    ma.rows = rows;
    ma.has_targets = targets != nullptr;
    ma.out = out;
    hipLaunchKernelGGL(head_stats_merge_kernel, dim3(1), dim3(256), 0, st, ma);
    HIPC(hipGetLastError());
    return BILD_OK;
}

int check_args(const bild_model* m, const float* x, int rows, bild_row_stats* out) {
    if (!m || !x || !out || rows < 1 || rows > kMaxRows) return BILD_EINVAL;
    if (((uintptr_t)x & 15) != 0) return BILD_EINVAL;  // rows are read with 16-byte loads
    return BILD_OK;
}

}  // namespace

extern "C" int bild_head_stats(const bild_model* m, const float* x_dev, int rows, const int32_t* targets_dev,
                               bild_row_stats* out_dev, void* hip_stream) {
    if (int rc = check_args(m, x_dev, rows, out_dev)) return rc;
    if (kernels_init() != hipSuccess) return BILD_EHIP;
    hipStream_t st = (hipStream_t)hip_stream;
    GemmArgs g = head_gemm(m, x_dev, rows, targets_dev, nullptr);
    const size_t bytes = kHdrBytes + gemm_num_blocks(g) * sizeof(StatPart) * kMaxRows;
    void* scr = nullptr;
    if (hipMalloc(&scr, bytes) != hipSuccess) return BILD_ENOMEM;
    g = head_gemm(m, x_dev, rows, targets_dev, scr);
    int rc = head_stats_run(m, x_dev, rows, targets_dev, out_dev, st, scr, g);
    if (hipStreamSynchronize(st) != hipSuccess && rc == BILD_OK) rc = BILD_EHIP;  // the scratch is in use until here
    (void)hipFree(scr);
    return rc;
}

extern "C" int bild_head_stats_static(const bild_model* m, const float* x_dev, int rows, const int32_t* targets_dev,
                                      bild_row_stats* out_dev, void* hip_stream) {
    if (int rc = check_args(m, x_dev, rows, out_dev)) return rc;
    if (kernels_init() != hipSuccess) return BILD_EHIP;
    void* scr = nullptr;
    if (int rc = scratch_of_device(&scr)) return rc;
    const GemmArgs g = head_gemm(m, x_dev, rows, targets_dev, scr);
    if ((int)gemm_num_blocks(g) > kStaticMaxParts) return BILD_ECAP;  // more partial statistics than the array holds
    return head_stats_run(m, x_dev, rows, targets_dev, out_dev, (hipStream_t)hip_stream, scr, g);
}
