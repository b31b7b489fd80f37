// The whole block-decode step as ONE persistent kernel.
//
// One workgroup per compute unit runs every phase of the step - embedding
// gather, then per layer QKV projection (+RoPE), shared-KV multi-draft
// attention, output projection (+residual), gate/up projection (+SwiGLU), down
// projection (+residual), and finally the LM head with its softmax statistics
// and the threshold unmask - separated by grid-wide barriers.  What makes this
// worth it in a memory-bound step: weights do not depend on the previous phase,
// so before a workgroup waits at a barrier it already issues the loads of the
// first weight tiles of the NEXT projection into its register ring.  The HBM
// stream therefore keeps running through barriers and through the short phases
// (attention, reductions) instead of draining at every kernel boundary.
//
// Barriers are monotonic counters in device memory: arrive with a release
// (write-back of this XCD's L2), spin with relaxed loads, then one acquire
// (invalidate) so the rows written by other XCDs are seen.  All workgroups must
// be co-resident, which the cooperative launch guarantees; a spin limit makes
// every wave exit even if that were violated (the status word then reports it).
#include "attn_core.h"
#include "gemm_core.h"
#include "rows_core.h"

namespace odb {

constexpr unsigned kSpinLimit = 1u << 21;      // ~ seconds; a healthy barrier needs a few polls

// Grid barrier without read-modify-write traffic: workgroup w publishes the barrier's epoch in
// flags[w]; the first wave of every workgroup polls all flags with one load per lane group.
// (Atomic increments of one shared counter from 256 workgroups on 8 XCDs serialise at the memory
// side and cost tens of microseconds per barrier.)  Epochs only grow, so flags need no reset.
struct Trace { unsigned long long *buf; unsigned idx; };     // optional timestamps (arrive, leave) per barrier

__device__ __forceinline__ void grid_sync(unsigned *flags, unsigned &epoch, int wg, int nwg, unsigned *status,
                                          Trace &tr) {
    if (tr.buf && threadIdx.x == 0) tr.buf[tr.idx++] = wall_clock64();
    __syncthreads();
    epoch += 1;
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        if (lane == 0) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            __hip_atomic_store(flags + wg, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        unsigned spins = 0;
        for (;;) {
            bool ok = true;
            for (int i = lane; i < nwg; i += 64) {
                unsigned v = __hip_atomic_load(flags + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = ok && (int)(v - epoch) >= 0;
            }
            if (__all(ok)) break;
            __builtin_amdgcn_s_sleep(1);
            if (++spins > kSpinLimit || __hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                if (lane == 0) __hip_atomic_store(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    __syncthreads();
    if (tr.buf && threadIdx.x == 0) tr.buf[tr.idx++] = wall_clock64();
}

// Returns x through an empty asm so that address arithmetic derived from it is redone in every
// phase instead of being hoisted out of the layer loop and kept in registers for the whole kernel.
__device__ __forceinline__ int opaque(int x) {
    asm volatile("" : "+s"(x));
    return x;
}

template <int MT, int PF, int DH>
__global__ __launch_bounds__(64 * WK) void step_kernel(StepArgs a) {
    __shared__ __attribute__((aligned(16))) char smem[kGemmSmemBytes];
    static_assert(attn_smem_bytes<1, WK>() <= kGemmSmemBytes, "LDS budget");
    const int wg0 = blockIdx.x, nwg = gridDim.x;
    unsigned target = a.barrier_base;
    Trace tr{a.trace ? a.trace + (size_t)wg0 * a.trace_stride : nullptr, 0};
    const int d = a.d, F = a.F, mt = a.mt_total;
    const int n_ssq = d / 16;
    const int lm_groups = (a.V / 16 + 2) / 3, lm_wgs = lm_groups < nwg ? lm_groups : nwg;   // as the stand-alone launch
    const float sc = 1.4426950408889634f * rsqrtf((float)DH);

    GemmArgs gq{a.hb, a.wqkv, d / 32, mt, 3 * d / 16, a.ssq, n_ssq, a.eps, 1.0f / (float)d};
    GemmArgs go{a.ao, a.wo, d / 32, mt, d / 16, nullptr, 0, 0.f, 0.f};
    GemmArgs gg{a.hb, a.wgu, d / 32, mt, 2 * F / 16, a.ssq, n_ssq, a.eps, 1.0f / (float)d};
    GemmArgs gd{a.act, a.wd, F / 32, mt, d / 16, nullptr, 0, 0.f, 0.f};

    frag_t w3[PF][3], w1[PF][1];
    gemm_prefetch_w<3, PF, WK, true>(gq, wg0, nwg, w3);

    // embedding gather (+ input of the first RMSNorm)
    for (int r = wg0; r < mt * 16; r += nwg)
        embed_row(r, a.embed, a.tokens, a.rm, d, a.V, a.h, NormOut{a.hb, a.ssq, a.g1, n_ssq}, mt);
    grid_sync(a.barrier, target, wg0, nwg, a.status, tr);

    for (int l = 0; l < a.n_layers; l++) {
        int wg = opaque(wg0);
        // QKV projection, RoPE, scatter into the attention layouts
        QkvOut qo = a.qo;
        gemm_wg<MT, 3, PF, true, EpiQKV, WK, true>(gq, EpiQKV{qo, mt}, wg, nwg, 0, w3, smem);
        grid_sync(a.barrier, target, wg0, nwg, a.status, tr);
        wg = opaque(wg0);

        // attention: one (row tile, head) per workgroup
        AttnArgs at = a.attn;
        at.kc += (size_t)l * a.cache_layer_stride;
        at.vc += (size_t)l * a.cache_layer_stride;
        for (int item = wg; item < mt * a.H; item += nwg) attn_wg<DH, 1, WK>(at, sc, item / a.H, item % a.H, smem);
        gemm_prefetch_w<1, PF>(go, wg, nwg, w1);
        grid_sync(a.barrier, target, wg0, nwg, a.status, tr);
        wg = opaque(wg0);

        // output projection + residual (+ input of the second RMSNorm)
        gemm_wg<MT, 1, PF, true>(go, EpiResid{a.h, d, NormOut{a.hb, a.ssq, a.g2 + (size_t)l * d, n_ssq}, mt}, wg, nwg, 0, w1,
                                 smem);
        gemm_prefetch_w<3, PF, WK, true>(gg, wg, nwg, w3);
        grid_sync(a.barrier, target, wg0, nwg, a.status, tr);
        wg = opaque(wg0);

        // gate/up projection + SiLU(gate)*up
        gemm_wg<MT, 3, PF, true, EpiSwiGLU, WK, true>(gg, EpiSwiGLU{a.act, mt}, wg, nwg, 0, w3, smem);
        gemm_prefetch_w<1, PF>(gd, wg, nwg, w1);
        grid_sync(a.barrier, target, wg0, nwg, a.status, tr);
        wg = opaque(wg0);

        // down projection + residual (+ input of the next layer's first RMSNorm, or of the final one)
        const bool last = l + 1 == a.n_layers;
        const float *gnext = last ? a.gf : a.g1 + (size_t)(l + 1) * d;
        gemm_wg<MT, 1, PF, true>(gd, EpiResid{a.h, d, NormOut{a.hb, a.ssq, gnext, n_ssq}, mt}, wg, nwg, 0, w1, smem);
        gq.W += a.qkv_stride; go.W += a.o_stride; gg.W += a.gu_stride; gd.W += a.d_stride;
        if (last) {
            gq = GemmArgs{a.hb, a.wlm, d / 32, mt, a.V / 16, a.ssq, n_ssq, a.eps, 1.0f / (float)d};
            gemm_prefetch_w<3, PF, WK, true>(gq, wg < lm_wgs ? wg : lm_wgs - 1, lm_wgs, w3);
        } else {
            gemm_prefetch_w<3, PF, WK, true>(gq, wg, nwg, w3);
        }
        grid_sync(a.barrier, target, wg0, nwg, a.status, tr);
    }

    // LM head: softmax statistics per (row, 16 vocabulary columns), then the per-draft finish
    if (wg0 < lm_wgs) gemm_wg<MT, 3, PF, true, EpiLMStats<MT / 2>, WK, true>(gq, EpiLMStats<MT / 2>(a.stats, lm_wgs * 3), wg0, lm_wgs, 0, w3, smem);
    grid_sync(a.barrier, target, wg0, nwg, a.status, tr);
    for (int u = wg0; u < a.rm.units; u += nwg) {
        __syncthreads();
        lm_finish_wg(u, a.stats, lm_wgs * 3, a.rm.units * a.rm.valid, a.rm.valid, a.rm.rpu_pad, a.tokens, a.mask_id, a.tau,
                     a.conf, a.argmax, a.unmask, reinterpret_cast<float *>(smem));
    }
}

size_t step_kernel_max_wgs(int device) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return 0;
    return (size_t)prop.multiProcessorCount;
}

template <int MT, int PF, int DH>
static hipError_t launch_one(const StepArgs &a, int nwg, hipStream_t s) {
    StepArgs copy = a;
    void *params[] = {&copy};
    return hipLaunchCooperativeKernel(reinterpret_cast<const void *>(&step_kernel<MT, PF, DH>), dim3(nwg), dim3(64 * WK),
                                      params, 0, s);
}

bool step_kernel_supports(const StepArgs &a) { return a.mt_total <= 8; }

hipError_t launch_step_kernel(const StepArgs &a, int nwg, hipStream_t s) {
    const bool pf_ok = (a.d / 32 / WK) % 4 == 0 && (a.F / 32 / WK) % 4 == 0;
    const bool pf2_ok = (a.d / 32 / WK) % 2 == 0 && (a.F / 32 / WK) % 2 == 0;
    if (a.mt_total <= 2) {
        if (a.dh == 128) return pf_ok ? launch_one<2, 4, 128>(a, nwg, s) : launch_one<2, 1, 128>(a, nwg, s);
        return pf_ok ? launch_one<2, 4, 64>(a, nwg, s) : launch_one<2, 1, 64>(a, nwg, s);
    }
    if (a.dh == 128) return pf2_ok ? launch_one<8, 2, 128>(a, nwg, s) : launch_one<8, 1, 128>(a, nwg, s);
    return pf2_ok ? launch_one<8, 2, 64>(a, nwg, s) : launch_one<8, 1, 64>(a, nwg, s);
}

}  // namespace odb
