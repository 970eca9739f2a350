// Persistent pass kernel: one launch runs a whole forward pass (embedding, every kept sublayer, LM head,
// greedy choice / accept) on a grid that is resident all at once; between dependent steps the workgroups
// meet at a grid barrier instead of ending a kernel.  Each step is the same block function the per-step
// kernels call, looped over that step's virtual blocks, so both paths produce identical bits.
//
// Data exchanged between workgroups inside the kernel is written and read with device-scope relaxed
// atomics (the per-XCD L2 caches are not coherent with each other); the barrier itself is an arrival
// counter hierarchy that only grows, polled with a bounded spin: a barrier that
// does not complete sets an error flag and lets every wave run on to the end, so the grid always drains.
#pragma once
#include "asd_attn.h"
#include "asd_gemm.h"
#include "asd_misc.h"

enum { OP_EMBED = 0, OP_QKV = 1, OP_ATTN = 2, OP_OPROJ = 3, OP_GU = 4, OP_DOWN = 5, OP_LM = 6, OP_FINISH = 7 };

struct PassOp {
    int32_t type;
    int32_t grid;        // virtual blocks of a GEMM step
    int32_t cls;         // ASD_K_* class (profiling / byte accounting on the host)
    int32_t pad;
    double bytes;        // algorithmic bytes of the step (host bookkeeping)
    GemmArgs g;
    AttnArgs t;
};

struct PassArgs {
    const PassOp* ops;
    int32_t n_ops;
    int32_t M, RS, d;
    const void* E;
    const int32_t* tokens;
    const float* g_first;
    float* xres;
    void* xb;
    int64_t xb_plane;
    float* part;
    const AmaxCand* cand;
    int32_t P_lm;
    int32_t fin_mode, fin_arg;
    int32_t* argmax;
    DevState* st;
    int32_t* tokbuf;
    int32_t* out;
    unsigned long long* bar;       // barrier words (see grid_sync), never reset
    unsigned long long bar_base;   // barriers completed before this launch
    int32_t* err;
};

#define PASS_THREADS 512
#define PASS_SPIN_LIMIT (1 << 20)

// Two-level barrier: workgroups arrive on one of BAR_GROUPS group counters (own cache lines); the last of a
// group arrives on the top counter; the workgroup that completes the top counter publishes the new epoch in
// every group's release word, which is what the group's members poll.  All counters only grow.
//   bar[0]                      top arrivals
//   bar[16 * (1 + g)]           arrivals of group g
//   bar[16 * (1 + BAR_GROUPS + g)]   release epoch of group g
#define BAR_GROUPS 8
__device__ __forceinline__ void grid_sync(unsigned long long* bar, unsigned long long epoch, int32_t* err) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);                 // this wave's stores (all write-through) have completed
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned G = gridDim.x, g = blockIdx.x % BAR_GROUPS;
        const unsigned gsize = G / BAR_GROUPS + (g < G % BAR_GROUPS ? 1u : 0u);
        unsigned long long* garr = bar + 16 * (1 + g);
        unsigned long long* grel = bar + 16 * (1 + BAR_GROUPS + g);
        const unsigned long long old = __hip_atomic_fetch_add(garr, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old + 1 == epoch * gsize) {            // last of the group
            const unsigned long long t = __hip_atomic_fetch_add(bar, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (t + 1 == epoch * BAR_GROUPS)       // last group: release everyone
                for (int q = 0; q < BAR_GROUPS; ++q)
                    __hip_atomic_store(bar + 16 * (1 + BAR_GROUPS + q), epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        int spins = 0;
        while (__hip_atomic_load(grel, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < epoch) {
            __builtin_amdgcn_s_sleep(4);
            if (++spins > PASS_SPIN_LIMIT) { *err = 1; break; }
        }
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

template <class T, int H>
__global__ __launch_bounds__(PASS_THREADS, 4) void pass_kernel(const PassArgs P) {
    __shared__ float red[PASS_THREADS];
    __shared__ int win[16];
    __shared__ float att_so[(PASS_THREADS / 64) * ATT_RH * H];
    __shared__ float att_ml[(PASS_THREADS / 64) * ASD_ROWS * 2];
    __shared__ unsigned att_old[PASS_THREADS / 64 / ATT_GW];
    using El = typename T::elem;
    const int wg = blockIdx.x, G = gridDim.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    constexpr int NWV = PASS_THREADS / 64;
    unsigned long long epoch = P.bar_base;
    for (int i = 0; i < P.n_ops; ++i) {
        const PassOp& op = P.ops[i];
        switch (op.type) {
            case OP_EMBED:
                for (int vb = wg; vb < EMBED_SPLIT * P.M; vb += G)
                    embed_block<T, true>((const El*)P.E, P.tokens, P.d, P.g_first, P.xres, P.xb, (size_t)P.xb_plane, P.RS, P.part,
                                         vb % EMBED_SPLIT, vb / EMBED_SPLIT, red);
                break;
            case OP_QKV:
                for (int vb = wg; vb < op.grid; vb += G) { gemm_block<T, EPI_QKV, 1, NWV, 4, true, T::NP == 2>(op.g, vb); __syncthreads(); }
                break;
            case OP_OPROJ:
            case OP_DOWN:
                for (int vb = wg; vb < op.grid; vb += G) { gemm_block<T, EPI_RES, 1, NWV, 4, true, T::NP == 2>(op.g, vb); __syncthreads(); }
                break;
            case OP_GU:
                for (int vb = wg; vb < op.grid; vb += G) { gemm_block<T, EPI_GU, 1, NWV, 4, true, T::NP == 2>(op.g, vb); __syncthreads(); }
                break;
            case OP_LM:
                for (int vb = wg; vb < op.grid; vb += G) { gemm_block<T, EPI_LM, 2, NWV, 4, true, T::NP == 2>(op.g, vb); __syncthreads(); }
                break;
            case OP_ATTN: {
                // two groups of ATT_GW waves per workgroup; every wave makes the same number of trips (the group
                // function synchronises the workgroup), idle groups pass valid = false
                constexpr int GPW = NWV / ATT_GW;
                const int last = op.t.st->pos + op.t.pos_off + op.t.M - 1;
                const int ng = last / ATT_GROUP + 1, units = ng * op.t.n_h;
                const int half = w / ATT_GW, hw = w % ATT_GW;
                for (int base = 0; base < units; base += G * GPW) {
                    const int u = base + half * G + wg;
                    const bool valid = u < units;
                    attn_group<T, H, true>(op.t, valid ? u % ng : 0, valid ? u / ng : 0, valid, hw, lane,
                                           att_so + (size_t)half * ATT_GW * ATT_RH * H, att_ml + half * ATT_GW * ASD_ROWS * 2, att_old + half);
                }
                break;
            }
            case OP_FINISH:
                if (wg == 0)
                    finish_block<true>(P.cand, P.P_lm, P.M, P.argmax, P.fin_mode, P.fin_arg, P.st, P.tokbuf, P.out, win);
                break;
        }
        if (i + 1 < P.n_ops) { epoch += 1; grid_sync(P.bar, epoch, P.err); }
    }
}
