// Dataflow pass kernel: one launch runs a whole forward pass (embedding, every kept sublayer, LM head, greedy
// choice / accept).  The grid is the concatenation of the steps' workgroups in step order; a workgroup runs the
// same block function as the per-step kernels, so both paths produce identical bits.
//
// Why: a batch-1 pass is a chain of ~5 dependent steps per layer, and a kernel boundary between two of them costs
// ~3 us of drain, cache write-back / invalidate and ramp-up during which nothing is requested from HBM.  Here the
// consumer's workgroups are dispatched while the producer's last ones still run (workgroups are dispatched in index
// order as slots free up), request the first ring of their weight fragments at once, and wait for their producer
// on a completion counter.
//
// No deadlock: a workgroup waits only for workgroups with LOWER indices, and those were dispatched before it, so
// they are running or done, and they in turn wait only for still lower ones.  Every wait is bounded all the same: a
// wait that gives up raises an error flag and lets the workgroup run on (with wrong data), so the grid always drains.
//
// Exchange between workgroups of the launch:
//   * a step's outputs are written with device-scope write-through stores (COH = true in the block functions);
//   * every buffer written inside the launch is written ONCE per launch and read only after its producer's
//     counter is complete (single assignment: each step has its own output buffers), so plain cached loads cannot
//     meet a stale line: no workgroup of this launch has touched the address before, and lines of an earlier
//     launch are invalidated at the kernel boundary;
//   * a producer workgroup bumps its step's counter after its stores have completed (wait for the wave's stores,
//     workgroup barrier, one device-scope atomic add).  Counters are sharded by physical XCD (workgroup index mod 8)
//     so that a step whose workgroups finish together does not serialise 256 increments on one address; a consumer
//     polls the eight shards with one load instruction;
//   * the last workgroup of the pass (the greedy choice) runs after every other one has bumped its counter, hence
//     after every wait has ended, and clears the counters for the next launch.
#pragma once
#include "asd_attn.h"
#include "asd_gemm.h"
#include "asd_misc.h"

enum { OP_EMBED = 0, OP_QKV = 1, OP_ATTN = 2, OP_OPROJ = 3, OP_GU = 4, OP_DOWN = 5, OP_LM = 6, OP_FINISH = 7 };

#define FLOW_THREADS 512
#define FLOW_WAVES (FLOW_THREADS / 64)
#define FLOW_SHARDS 8                   // counter shards per step = XCDs
#define FLOW_SHARD_WORDS 16             // 64 bytes per shard counter
#define FLOW_SPIN_LIMIT (1 << 20)

struct PassOp {
    int32_t type;
    int32_t grid;        // workgroups of the step that do work (per-step kernels: the launch's grid)
    int32_t cls;         // ASD_K_* class (profiling / byte accounting on the host)
    int32_t tn;          // dataflow kernel: weight tiles per workgroup of a GEMM step
    double bytes;        // algorithmic bytes of the step (host bookkeeping)
    // dataflow kernel
    int32_t first_block; // index of the step's first workgroup in the pass's grid (a multiple of 8)
    int32_t n_blocks;    // workgroups the step occupies in the grid (grid rounded up to a multiple of 8; the extra ones only signal)
    int32_t dep;         // step whose completion this step waits for (-1: none)
    int32_t dep_target[FLOW_SHARDS];   // workgroups of step `dep` per counter shard
    GemmArgs g;
    AttnArgs t;
};

struct FlowArgs {
    const PassOp* ops;
    const uint16_t* op_of_block;   // [grid]
    int32_t n_ops;
    int32_t M, RS, d, vocab;
    const void* E;
    const int32_t* tokens;
    const float* g_first;
    float* xres0;                  // embedding output: residual stream, tiled normed copy, ||x||^2 partials
    void* xb0;
    int64_t xb_plane;
    float* part0;
    const AmaxCand* cand;
    int32_t P_lm;
    int32_t fin_mode, fin_arg;
    int32_t* argmax;
    DevState* st;
    int32_t* tokbuf;
    int32_t* out;
    unsigned* done;                // [n_ops][FLOW_SHARDS][FLOW_SHARD_WORDS] completion counters, zero between launches
    int32_t* err;
};

// Block until step op.dep is complete.  Called by every thread of the workgroup.
__device__ __forceinline__ void flow_wait(const FlowArgs& P, const PassOp& op) {
    if (op.dep >= 0) {
        if (threadIdx.x < 64) {
            const int lane = threadIdx.x;
            const unsigned target = lane < FLOW_SHARDS ? (unsigned)op.dep_target[lane & (FLOW_SHARDS - 1)] : 0u;
            const unsigned* p = P.done + ((size_t)op.dep * FLOW_SHARDS + (lane & (FLOW_SHARDS - 1))) * FLOW_SHARD_WORDS;
            int spins = 0;
            for (;;) {
                const unsigned v = lane < FLOW_SHARDS ? __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
                if (__all(v >= target)) break;
                __builtin_amdgcn_s_sleep(1);
                if (++spins > FLOW_SPIN_LIMIT) { if (lane == 0) *P.err = 1; break; }
            }
        }
        __syncthreads();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    }
}

// This workgroup's part of step oi is done: its stores have completed, then the step's counter shard is bumped.
__device__ __forceinline__ void flow_signal(const FlowArgs& P, const int oi) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);                 // this wave's stores (write-through) have completed
    __syncthreads();
    if (threadIdx.x == 0)
        __hip_atomic_fetch_add(P.done + ((size_t)oi * FLOW_SHARDS + (blockIdx.x & (FLOW_SHARDS - 1))) * FLOW_SHARD_WORDS, 1u, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
}

template <class A, class B> constexpr size_t flow_max(A a, B b) { return (size_t)a > (size_t)b ? (size_t)a : (size_t)b; }

template <class T, int H, bool PACK>
__global__ __launch_bounds__(FLOW_THREADS, 4) void flow_kernel(const FlowArgs P) {
    constexpr int NW = FLOW_WAVES, U = 4, GPW = NW / ATT_GW;
    using LQ = GemmLds<T, EPI_QKV, 1, NW, PACK>;
    using LR1 = GemmLds<T, EPI_RES, 1, NW, PACK>;
    using LR2 = GemmLds<T, EPI_RES, 2, NW, PACK>;
    using LG = GemmLds<T, EPI_GU, 1, NW, PACK>;
    using LL = GemmLds<T, EPI_LM, 2, NW, PACK>;
    struct AttLds { float so[GPW][ATT_GW * ATT_RH * H]; float sml[GPW][ATT_GW * ASD_ROWS * 2]; unsigned old[GPW]; };
    struct MiscLds { float red[EMBED_THREADS]; int win[16]; };
    constexpr size_t LDS_BYTES = flow_max(flow_max(flow_max(sizeof(LQ), sizeof(LR1)), flow_max(sizeof(LR2), sizeof(LG))),
                                          flow_max(flow_max(sizeof(LL), sizeof(AttLds)), sizeof(MiscLds)));
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
    using El = typename T::elem;

    const int b = blockIdx.x, tid = threadIdx.x;
    const int oi = P.op_of_block[b];
    const PassOp& op = P.ops[oi];
    const int vb = b - op.first_block;
    auto dep = [&]() { flow_wait(P, op); };

    if (vb < op.grid) {
        switch (op.type) {
            case OP_EMBED:
                embed_block<T, true>((const El*)P.E, P.tokens, P.d, P.vocab, P.st, P.g_first, P.xres0, P.xb0, (size_t)P.xb_plane, P.RS, P.part0,
                                     vb % EMBED_SPLIT, vb / EMBED_SPLIT, reinterpret_cast<MiscLds*>(lds)->red);
                break;
            // (the step's arguments are copied out of the table first: read through the table they would be re-read
            // after every store, which the compiler must assume may alias them)
            case OP_QKV: {
                const GemmArgs g = op.g;
                gemm_block<T, EPI_QKV, 1, NW, U, true, PACK>(g, vb, *reinterpret_cast<LQ*>(lds), dep);
                break;
            }
            case OP_OPROJ:
            case OP_DOWN: {
                const GemmArgs g = op.g;
                if (op.tn == 2) gemm_block<T, EPI_RES, 2, NW, U, true, PACK>(g, vb, *reinterpret_cast<LR2*>(lds), dep);
                else gemm_block<T, EPI_RES, 1, NW, U, true, PACK>(g, vb, *reinterpret_cast<LR1*>(lds), dep);
                break;
            }
            case OP_GU: {
                const GemmArgs g = op.g;
                gemm_block<T, EPI_GU, 1, NW, U, true, PACK>(g, vb, *reinterpret_cast<LG*>(lds), dep);
                break;
            }
            case OP_LM: {
                const GemmArgs g = op.g;
                gemm_block<T, EPI_LM, 2, NW, U, true, PACK>(g, vb, *reinterpret_cast<LL*>(lds), dep);
                break;
            }
            case OP_ATTN: {
                // two groups of ATT_GW waves per workgroup; both make the same calls (the group function
                // synchronises the workgroup), a padding unit passes valid = false
                AttLds* L = reinterpret_cast<AttLds*>(lds);
                const AttnArgs t = op.t;
                const int w = __builtin_amdgcn_readfirstlane(tid >> 6), half = w / ATT_GW, hw = w % ATT_GW;
                int grp = 0, head = 0;
                const bool valid = attn_unit(t, vb * GPW + half, &grp, &head);
                dep();
                attn_group<T, H, true>(t, valid ? grp : 0, valid ? head : 0, valid, hw, tid & 63, L->so[half], L->sml[half], &L->old[half]);
                break;
            }
            case OP_FINISH: {
                dep();
                finish_block<true>(P.cand, P.P_lm, P.M, P.vocab, P.argmax, P.fin_mode, P.fin_arg, P.st, P.tokbuf, P.out,
                                   reinterpret_cast<MiscLds*>(lds)->win);
                // every other workgroup of the pass has bumped its counter (the steps form a chain that ends here), so no
                // wait is still in progress: clear the counters for the next launch
                for (int i = tid; i < P.n_ops * FLOW_SHARDS; i += FLOW_THREADS)
                    __hip_atomic_store(P.done + (size_t)i * FLOW_SHARD_WORDS, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                return;
            }
        }
    }
    flow_signal(P, oi);
}
