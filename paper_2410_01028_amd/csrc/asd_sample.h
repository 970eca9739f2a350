// Sampled decoding (temperature > 0): token draws and the speculative-sampling verification.
//
// Section 1 cites the speculative-sampling rule for sampled decoding (temperatures 0.2 and 0.6 in the
// experiments) without printing it; this is that published rule.  A draft token x ~ q is kept with
// probability min(1, p(x)/q(x)); the first rejected draft is replaced by a draw from the normalised
// residual max(0, p - q); when every draft is kept one more token is drawn from the full model's next
// distribution.  q and p are softmax(logits / T) of the draft and the full model.
//
// Uniforms are counter based, so a run is reproducible and independent of how cycles fall:
//   U(e, c) = (mix64(stream + (3e + c + 1) * GOLD) >> 11) * 2^-53 for output index e and purpose c
//   (0 draft draw, 1 accept test, 2 replacement / extra / plain draw).
// Each kernel is one workgroup of SAMPLE_THREADS threads; every reduction has a fixed order (thread-contiguous
// segments, then a tree over the threads), decisions are taken in double on fp32 weights.
#pragma once
#include "asd_common.h"
#include "asd_misc.h"

#define SAMPLE_THREADS 1024

struct SampleArgs {
    const float* logits;     // [rows][V] logits of the pass just finished
    float* qlogits;          // [draft steps][V] draft-model logits kept until the verification
    double* qstat;           // [draft steps][2] their softmax statistics (maximum, Z), left by the draft draws
    int32_t V;
    float inv_T;
    uint64_t stream;         // key of the sampling stream (from the seed)
    DevState* st;
    int32_t* tokbuf;
    int32_t* out;
};

__device__ __forceinline__ double sample_uniform(uint64_t stream, int64_t index, int purpose) {
    const uint64_t G = 0x9E3779B97F4A7C15ULL;
    const uint64_t c = (uint64_t)(3 * index + purpose);
    return (double)(mix64(stream + (c + 1) * G) >> 11) * (1.0 / 9007199254740992.0);
}

// fixed-order block reductions over one value per thread; every thread gets the result
__device__ __forceinline__ float blk_max(float v, float* red) {
    const int tid = threadIdx.x;
    red[tid] = v;
    __syncthreads();
    for (int s = SAMPLE_THREADS / 2; s > 0; s >>= 1) {
        if (tid < s) red[tid] = fmaxf(red[tid], red[tid + s]);
        __syncthreads();
    }
    const float r = red[0];
    __syncthreads();
    return r;
}
__device__ __forceinline__ double blk_sum(double v, double* red) {
    const int tid = threadIdx.x;
    red[tid] = v;
    __syncthreads();
    for (int s = SAMPLE_THREADS / 2; s > 0; s >>= 1) {
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    const double r = red[0];
    __syncthreads();
    return r;
}

// A thread's share of a row of V values is the contiguous segment [lo, lo + n), n <= seg = ceil(V / SAMPLE_THREADS).
// SEG > 0: the segment is held in registers, padded to SEG values with -inf (seg <= SEG; one pass over memory per
// row, all loads in flight at once; a single workgroup walking memory element by element spends its time on load latency).  SEG = 0: the
// segment is read from memory at every use (any V).  Both run the same arithmetic in the same order.
#define SAMPLE_SEG 32                     // register path: V <= SAMPLE_SEG * SAMPLE_THREADS

template <int SEG>
struct RowSeg {
    const float* row;                     // the row in memory
    int lo, n;
    float v[SEG > 0 ? SEG : 1];
    __device__ __forceinline__ void load(const float* r, int V) {
        const int seg = (V + SAMPLE_THREADS - 1) / SAMPLE_THREADS;
        row = r; lo = min(V, (int)threadIdx.x * seg); n = min(V, lo + seg) - lo;
        if constexpr (SEG > 0) {
#pragma unroll
            for (int k = 0; k < SEG; ++k) v[k] = k < n ? r[lo + k] : -INFINITY;
        }
    }
    // f(k, value) for k = 0 .. n-1 in ascending order.  The register variant also calls f for the padding
    // k = n .. SEG-1 with value -inf (no branches): a logit of -inf leaves a maximum, a sum of exponentials and a
    // running sum of weights exactly as they were.
    template <class F> __device__ __forceinline__ void each(F f) const {
        if constexpr (SEG > 0) {
#pragma unroll
            for (int k = 0; k < SEG; ++k) {
                f(k, v[k]);
                if (k % 4 == 3) __builtin_amdgcn_sched_barrier(0);       // (or the scheduler starts all SEG chains at once and spills)
            }
        } else {
            for (int k = 0; k < n; ++k) f(k, row[lo + k]);
        }
    }
};

// softmax statistics of a logit row at temperature 1/inv_T: the maximum and Z = sum exp((l - max) * inv_T)
template <int SEG>
__device__ __forceinline__ void row_stats(const RowSeg<SEG>& r, float inv_T, float* mx, double* Z, float* fred, double* dred) {
    float m = -INFINITY;
    r.each([&](int, float x) { m = fmaxf(m, x); });
    *mx = blk_max(m, fred);
    const float mxv = *mx;
    double s = 0.0;
    r.each([&](int, float x) { s += (double)expf((x - mxv) * inv_T); });
    *Z = blk_sum(s, dred);
}

// Inverse-CDF draw from the non-negative weights w(k, .) of the threads' segments (seg: the segment whose each()
// enumerates this thread's elements; w gets the local index and that segment's value): the smallest global index
// whose running sum exceeds u * total; if rounding leaves none, the last index with a positive weight.  Every
// thread returns the drawn index.
template <int SEG, class F>
__device__ __forceinline__ int blk_sample(const RowSeg<SEG>& seg, F w, double u, double* dred, int* ired) {
    const int tid = threadIdx.x;
    double s = 0.0;
    int last_pos = -1;
    seg.each([&](int k, float x) {
        const double wi = (double)w(k, x);
        s += wi;
        if (wi > 0.0) last_pos = seg.lo + k;
    });
    // inclusive scan over the threads' segment sums (Hillis-Steele in LDS, fixed order)
    dred[tid] = s;
    __syncthreads();
    for (int off = 1; off < SAMPLE_THREADS; off <<= 1) {
        const double add = tid >= off ? dred[tid - off] : 0.0;
        __syncthreads();
        dred[tid] += add;
        __syncthreads();
    }
    const double incl = dred[tid], total = dred[SAMPLE_THREADS - 1];
    const double excl = incl - s;
    __syncthreads();
    const double t = u * total;
    if (tid == 0) { ired[0] = -1; ired[1] = -1; }
    __syncthreads();
    if (last_pos >= 0) atomicMax(&ired[1], last_pos);
    if (incl > t && excl <= t && seg.n > 0) {
        double cum = excl;
        int pick = -1;
        seg.each([&](int k, float x) {
            cum += (double)w(k, x);
            if (pick < 0 && cum > t) pick = seg.lo + k;
        });
        if (pick < 0) pick = last_pos >= 0 ? last_pos : seg.lo + seg.n - 1;   // the segment's sum exceeded t, re-adding it did not: its last weight
        atomicMax(&ired[0], pick);          // one thread at most gets here with pick >= 0 (incl is non-decreasing)
    }
    __syncthreads();
    const int r = ired[0] >= 0 ? ired[0] : max(ired[1], 0);
    __syncthreads();
    return r;
}

// After a draft step: keep its logits for the verification and draw the draft token of output index
// index_base + emitted + j into row j+1 of the coming verification pass.
template <int SEG>
__global__ __launch_bounds__(SAMPLE_THREADS) void sample_draft_kernel(const SampleArgs a, int j) {
    __shared__ float fred[SAMPLE_THREADS];
    __shared__ double dred[SAMPLE_THREADS];
    __shared__ int ired[2];
    const float* lg = a.logits;
    float* keep = a.qlogits + (size_t)j * a.V;
    for (int i = threadIdx.x; i < a.V; i += SAMPLE_THREADS) keep[i] = lg[i];
    RowSeg<SEG> r;
    r.load(lg, a.V);
    float mx; double Z;
    row_stats(r, a.inv_T, &mx, &Z, fred, dred);
    const double u = sample_uniform(a.stream, (int64_t)a.st->index_base + a.st->emitted + j, 0);
    const float inv_T = a.inv_T;
    const int tok = blk_sample(r, [&](int, float x) { return expf((x - mx) * inv_T); }, u, dred, ired);
    if (threadIdx.x == 0) { a.tokbuf[j + 1] = tok; a.qstat[2 * j] = (double)mx; a.qstat[2 * j + 1] = Z; }
}

// A plain draw (purpose 2) of output index `index` from logits row `row` into tokbuf[0]: the prompt pass's token.
template <int SEG>
__global__ __launch_bounds__(SAMPLE_THREADS) void sample_plain_kernel(const SampleArgs a, int row, int64_t index) {
    __shared__ float fred[SAMPLE_THREADS];
    __shared__ double dred[SAMPLE_THREADS];
    __shared__ int ired[2];
    RowSeg<SEG> r;
    r.load(a.logits + (size_t)row * a.V, a.V);
    float mx; double Z;
    row_stats(r, a.inv_T, &mx, &Z, fred, dred);
    const float inv_T = a.inv_T;
    const int tok = blk_sample(r, [&](int, float x) { return expf((x - mx) * inv_T); }, sample_uniform(a.stream, index, 2), dred, ired);
    if (threadIdx.x == 0) a.tokbuf[0] = tok;
}

// After a verification pass over rows [last, d_1 .. d_kk]: speculative-sampling accept / replace, then the same
// bookkeeping as the greedy accept step (emit, advance the cache length by a + 1, next first row).
template <int SEG>
__global__ __launch_bounds__(SAMPLE_THREADS) void sample_accept_kernel(const SampleArgs a, int kk) {
    __shared__ float fred[SAMPLE_THREADS];
    __shared__ double dred[SAMPLE_THREADS];
    __shared__ int ired[2];
    const int V = a.V;
    const float inv_T = a.inv_T;
    const int64_t e0 = (int64_t)a.st->index_base + a.st->emitted;
    int acc = kk, next = 0;
    for (int i = 0; i < kk; ++i) {
        const float* ql = a.qlogits + (size_t)i * V;
        const float* pl = a.logits + (size_t)i * V;
        RowSeg<SEG> rp;
        rp.load(pl, V);
        const int x = a.tokbuf[i + 1];
        // the draft row's statistics were left by its draw (same arithmetic on the same values)
        const float mq = (float)a.qstat[2 * i];
        const double Zq = a.qstat[2 * i + 1];
        float mp; double Zp;
        row_stats(rp, inv_T, &mp, &Zp, fred, dred);
        const double q = (double)expf((ql[x] - mq) * inv_T) / Zq, p = (double)expf((pl[x] - mp) * inv_T) / Zp;
        if (sample_uniform(a.stream, e0 + i, 1) * q < p) continue;          // kept (the same decision in every thread)
        // rejected (at most once per cycle): draw the replacement from the normalised residual, or from p should the
        // residual vanish.  Both rows are read from memory here: held in registers, the residual weights of the three
        // walks (sum, scan input, pick) are kept alive as one array of doubles and the kernel spills.
        const float iZq = (float)(1.0 / Zq), iZp = (float)(1.0 / Zp);
        RowSeg<0> rm;
        rm.load(pl, V);
        auto resid = [&](int k, float pv) { return fmaxf(0.f, expf((pv - mp) * inv_T) * iZp - expf((ql[rm.lo + k] - mq) * inv_T) * iZq); };
        double rs = 0.0;
        rm.each([&](int k, float pv) { rs += (double)resid(k, pv); });
        const double R = blk_sum(rs, dred);
        const double u = sample_uniform(a.stream, e0 + i, 2);
        next = R > 0.0 ? blk_sample(rm, resid, u, dred, ired)
                       : blk_sample(rm, [&](int, float pv) { return expf((pv - mp) * inv_T); }, u, dred, ired);
        acc = i;
        break;
    }
    if (acc == kk) {
        RowSeg<SEG> rp;
        rp.load(a.logits + (size_t)kk * V, V);
        float mp; double Zp;
        row_stats(rp, inv_T, &mp, &Zp, fred, dred);
        next = blk_sample(rp, [&](int, float pv) { return expf((pv - mp) * inv_T); }, sample_uniform(a.stream, e0 + kk, 2), dred, ired);
    }
    if (threadIdx.x != 0) return;
    DevState* st = a.st;
    int e = st->emitted;
    for (int q = 1; q <= acc && e < st->target; ++q) a.out[e++] = a.tokbuf[q];
    if (e < st->target) a.out[e++] = next;
    st->emitted = e;
    st->pos += acc + 1;
    st->cycles += 1; st->drafted += kk; st->accepted += acc;
    a.tokbuf[0] = next;
}
