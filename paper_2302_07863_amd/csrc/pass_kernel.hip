// Persistent decoder-pass kernel for gfx950.
//
// At the paper's model sizes (Table 2) one decoder layer holds a few tens of MB of weights,
// which the chip streams in a few microseconds; a pass made of one kernel launch per
// projection / attention then spends most of its time between kernels.  This kernel runs the
// embedding and every layer of a pass (Section 3.2: one row for the small model's step, n+1
// rows for the large model's review) in ONE launch: G workgroups of 8 waves stay resident,
// read the list of stages from device memory and meet at a grid barrier after each stage.
// The stage bodies are the same device functions the one-kernel-per-stage launches use.
//
// Barrier: one arrival counter that only grows.  A workgroup's base is the counter value at
// the end of the previous launch (PassSync::epoch, rewritten by workgroup 0 after the last
// barrier), so a captured launch replays without host-side arguments.  Everything one stage
// hands to the next (activations, new K/V rows) is written and read with agent-scope atomic
// accesses (COH = true in the bodies), so the barrier needs no cache-wide write-back or
// invalidate: each wave waits for its own stores, the workgroup meets, thread 0 adds 1 and
// polls until the counter reaches base + k*G, and the workgroup meets again.  A wait that
// exceeds `spin_limit` polls sets the fault flag, which every other waiter also polls, and
// all workgroups return: the kernel always ends.
#define BILD_DEVICE_ONLY
#include "kernels.hip"

#include <stddef.h>

namespace bild {

// The stage list does not change while a pass runs, so it is read through the constant address
// space: arguments then arrive by scalar loads whenever a stage body needs them, exactly like the
// kernel arguments of the one-kernel-per-stage launches, instead of occupying registers throughout.
#define BILD_CONST_AS __attribute__((address_space(4)))
typedef const BILD_CONST_AS Stage CStage;

// Stage bodies as functions of their own: each then gets the register allocation it has as a kernel,
// instead of one allocation over the union of all bodies inside the stage loop.
// weight tiles per load batch of a wave inside the persistent kernel
#ifndef BILD_RESIDENT_BATCH
#define BILD_RESIDENT_BATCH 8
#endif
constexpr int kResidentBatch = BILD_RESIDENT_BATCH;
#ifdef BILD_PASS_CALLS
#define BILD_UNIT __noinline__
#else
#define BILD_UNIT __forceinline__
#endif
template <int DT, int RW, int EPI, int ROPE, int NT>
__device__ BILD_UNIT void gemm_unit(const BILD_CONST_AS GemmArgs* a, int vb, char* smem) {
    gemm_body<DT, RW, EPI, ROPE, NT, kResidentBatch / RW, true>(*a, vb, smem);
}
template <int DT, int DH32>
__device__ BILD_UNIT void attn_unit(const BILD_CONST_AS AttnArgs* a, int vb, char* smem) {
    attn_body<DT, DH32, true>(*a, vb, smem);
}

template <int DT, int NT, int DH32>
__global__ __launch_bounds__(512) void pass_kernel(const PassArgs p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    __shared__ int s_quit;
    const int tid = threadIdx.x;
    const int G = (int)gridDim.x, wg = (int)blockIdx.x;
    unsigned target = __hip_atomic_load(&p.sync->epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tid == 0) s_quit = 0;
    __syncthreads();

#ifdef BILD_TRACE
#define PSTAMP(i) do { if (p.trace && tid == 0 && wg == p.trace_wg) p.trace[s * 8 + (i)] = wall_clock64(); } while (0)
#else
#define PSTAMP(i) do { } while (0)
#endif
    for (int s = 0; s < p.nstages; ++s) {
        CStage& st = *(CStage*)(p.prog + s);
        const int kind = st.kind, nb = st.nblocks;
        PSTAMP(0);
        if (kind == ST_GEMM) {
            for (int vb = wg; vb < nb; vb += G) {
                if (vb != wg) __syncthreads();  // the LDS of the previous unit is free again
                if (st.g.rw == 2)
                    gemm_unit<DT, 2, EPI_ACT, 0, NT>(&st.g, vb, smem);
                else
                    gemm_unit<DT, 1, -1, -1, NT>(&st.g, vb, smem);
            }
        } else if (kind == ST_ATTN) {
            for (int vb = wg; vb < nb; vb += G) {
                if (vb != wg) __syncthreads();
                attn_unit<DT, DH32>(&st.a, vb, smem);
            }
        } else if (kind == ST_ATTN_MERGE) {
            for (int vb = wg; vb < nb; vb += G) attn_merge_body<true>(st.a, vb);
        } else {  // ST_EMBED
            for (int vb = wg; vb < nb; vb += G) embed_body<DT, true>(st.e, vb);
        }
        PSTAMP(1);
        if (s + 1 == p.nstages) break;

        {   // touch the next stage's arguments: they are in the scalar cache when the barrier opens
            const BILD_CONST_AS int* nx = (const BILD_CONST_AS int*)(p.prog + s + 1);
            int warm = 0;
#pragma unroll
            for (int i = 0; i < (int)(sizeof(Stage) / 4); i += 16) warm ^= nx[i];
            asm volatile("" ::"s"(warm));
        }
        target += (unsigned)G;
        // every activation store of this workgroup has been performed at agent scope once its wave's
        // memory counters reach zero; the workgroup barrier then covers all waves
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        PSTAMP(2);
        if (tid == 0) {
            PSTAMP(3);
            __hip_atomic_fetch_add(&p.sync->arrivals, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            int polls = 0;
            while (true) {
                if (p.spin_limit >= 0) {  // a negative limit is the host forcing the give-up path (tests)
                    const unsigned seen = __hip_atomic_load(&p.sync->arrivals, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if ((int)(seen - target) >= 0) break;
                }
                const int bad = __hip_atomic_load(p.fault, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (bad || ++polls > p.spin_limit) {
                    __hip_atomic_store(p.fault, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    s_quit = 1;
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            PSTAMP(4);
            PSTAMP(5);
        }
        __syncthreads();
        PSTAMP(6);
        if (s_quit) return;  // uniform: every thread reads the same LDS word after the barrier
    }
#undef PSTAMP
    if (wg == 0 && tid == 0) __hip_atomic_store(&p.sync->epoch, target, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

#ifndef BILD_PASS_DT
#error "compile with -DBILD_PASS_DT=0 (fp32 models) or 1 (bf16 models)"
#endif
#define BILD_CAT2(a, b) a##b
#define BILD_CAT(a, b) BILD_CAT2(a, b)

template <int NT, int DH32>
static hipError_t launch_one(const PassArgs& p, int G, size_t lds, hipStream_t st) {
    hipLaunchKernelGGL((pass_kernel<BILD_PASS_DT, NT, DH32>), dim3(G), dim3(512), lds, st, p);
    return hipGetLastError();
}

// launch_pass_dt0 / launch_pass_dt1: the variants of one storage type (one translation unit each)
hipError_t BILD_CAT(launch_pass_dt, BILD_PASS_DT)(const PassArgs& p, int nt, int dh32, int G, size_t lds, hipStream_t st) {
    if (nt == 2)
        return dh32 == 1 ? launch_one<2, 1>(p, G, lds, st)
                         : (dh32 == 2 ? launch_one<2, 2>(p, G, lds, st) : launch_one<2, 4>(p, G, lds, st));
    return dh32 == 1 ? launch_one<1, 1>(p, G, lds, st)
                     : (dh32 == 2 ? launch_one<1, 2>(p, G, lds, st) : launch_one<1, 4>(p, G, lds, st));
}

// Function attributes of every variant; called once, before any stream capture.
hipError_t BILD_CAT(pass_kernels_init_dt, BILD_PASS_DT)(int lds_limit) {
    const void* fns[] = {(const void*)pass_kernel<BILD_PASS_DT, 1, 1>, (const void*)pass_kernel<BILD_PASS_DT, 1, 2>,
                         (const void*)pass_kernel<BILD_PASS_DT, 1, 4>, (const void*)pass_kernel<BILD_PASS_DT, 2, 1>,
                         (const void*)pass_kernel<BILD_PASS_DT, 2, 2>, (const void*)pass_kernel<BILD_PASS_DT, 2, 4>};
    for (const void* f : fns) {
        hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, lds_limit);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace bild
