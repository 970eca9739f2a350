// Weight-streaming small-M GEMM: out[m][n] = sum_k X[m][k] * W[n][k], m < 16, with fused epilogues.
//
// One workgroup owns a few 16-row tiles of W; its NW waves split K (contiguous slices, or
// interleaved k-blocks), each wave streaming its share of every tile (1 KiB per load
// instruction, U steps in flight) through the matrix cores with the 16 activation rows as
// the other operand.  The waves' sums are then added through LDS in wave order, so every
// output element has one fixed reduction order that does not depend on how many of the 16
// rows are in use: row i of a (k+1)-row verification pass and the same row run alone give
// identical bits.  The grid never depends on the row count either.
//
// Epilogues (what a decoder sublayer needs right after the contraction):
//   EPI_QKV  RMSNorm scale, rotary embedding, q -> tiled q buffer, k/v -> paged KV cache
//            (the fused QKV weight is tiled with each rotary pair's two rows in the same tile)
//   EPI_RES  y = x + out (residual add), tiled copy of y*gain for the next norm, and the
//            cosine tap: per-workgroup partials of <x,y> and ||y||^2
//   EPI_GU   RMSNorm scale, silu(gate) * up -> tiled activation
//   EPI_LM   RMSNorm scale, logits, per-workgroup argmax candidates and softmax partial sums
// The three epilogues that need the RMSNorm scale are always the next launch after an
// EPI_RES kernel (or after the embedding): every workgroup sums that kernel's partials in
// the same fixed order to get ||y||^2, and workgroup 0 also finishes the producing
// sublayer's cosine, cos = <x,y> / sqrt(||x||^2 ||y||^2).  No workgroup ever waits for
// another inside a kernel, so no device-scope fence (and no L2 write-back) is needed.
#pragma once
#include "asd_common.h"

enum { EPI_QKV = 0, EPI_RES = 1, EPI_GU = 2, EPI_LM = 3 };

struct AmaxPart { float v; int32_t i; float s; float pad; };   // best logit, its index, sum of exp(logit - v) over the workgroup's features

struct GemmArgs {
    const u32x4* W;          // tiled weights
    const u32x4* W2;         // EPI_GU: tiled up-projection (W is the gate projection)
    const u32x4* X;          // tiled activations (row stride RS; T::NP planes, x_plane fragments apart)
    int64_t x_plane;
    int32_t n_tiles;         // output features / 16
    int32_t KB;              // k-blocks
    int64_t w_tile_stride, w_kb_stride;   // fragment (KiB) strides of the weight layout: tile-major {KB, 1}, k-major {1, tiles}
    int32_t k_interleave;    // how the waves of a workgroup split K
    int32_t M;               // rows in use
    int32_t RS;              // row stride of every activation buffer in this pass (power of two >= M)
    float* ssq;              // [16] ||residual row||^2 as of the last finished cosine tap
    float inv_d, eps;
    // input side of QKV / GU / LM: partials of the kernel that produced the residual
    const float* part_in;    // [P_in][16][2]
    int32_t P_in;
    float* fin_cos_rows;     // [16] cosine per row of the producing sublayer (written by workgroup 0); NULL after the embedding
    double* fin_cos_acc;     // its running sum over rows
    // EPI_RES
    float* xres;             // [16][d] fp32 residual stream, updated in place
    void* xb;                // tiled copy of y * g_next in storage type
    int64_t xb_plane, q_plane, hmid_plane;   // plane strides (elements) of the activation buffers written here
    const float* g_next;     // gain of the norm that reads y next
    float* part;             // [grid][16][2] partial <x,y>, ||y||^2 of this workgroup's features
    int32_t d;
    // EPI_QKV
    const DevState* st;
    int32_t pos_off;
    const float* rope;       // [max_seq][h/2][2] cos, sin
    void* q;                 // [n_h][h/KE][RS][KE]
    void* kv;                // this layer's cache pages
    const int32_t* page_table;
    int32_t n_h, n_kv, h, page_tokens;
    // EPI_GU
    void* hmid;
    // EPI_LM
    float* logits;           // [16][V]
    int32_t V;
    AmaxPart* amax_part;     // [grid][16] best (logit, index) among this workgroup's features, and their exp-sum
};

// Stream n k-blocks kb = first, first + step, ... of NA weight tiles and the matching activation fragments
// (NPL fragments per k-block, xpl apart, each with its own accumulators).
// `between` runs after the first U steps have been requested: work whose own loads should overlap the stream.
// X points at this lane's fragment of k-block 0 (always a valid address); consecutive k-blocks are xstep fragments
// apart.
template <class T, int NA, int NPL, int U, class F>
__device__ __forceinline__ void stream_mma(const u32x4* const (&A)[NA], const u32x4* X, int xstep, int64_t xpl, int first, int step, int n,
                                           int64_t wks, f32x4 (&acc)[NPL][NA], F between) {
    // A ring of U slots.  The steady-state loop has no conditional request in it, and X is a valid address in every
    // lane (a lane whose row is not in use reads another row's fragment: its column of the products is never read,
    // and zeroing it would be a use that waits for the load).  The wait counts the compiler derives are exact only
    // when every path issues the same loads; a single request under a condition made it wait for ALL outstanding
    // loads at the top of every trip, which turns the ring into load-everything-then-drain.
    u32x4 a[U][NA], b[U][NPL];
    auto fill = [&](const int u, const int kb) {
#pragma unroll
        for (int pl = 0; pl < NPL; ++pl) b[u][pl] = *(X + (size_t)(first + kb * step) * xstep + pl * xpl);
#pragma unroll
        for (int s = 0; s < NA; ++s) a[u][s] = __builtin_nontemporal_load(A[s] + (size_t)(first + kb * step) * ASD_WAVE * wks);
    };
    auto use = [&](const int u) {
#pragma unroll
        for (int s = 0; s < NA; ++s)
#pragma unroll
            for (int pl = 0; pl < NPL; ++pl) mma16<T>(acc[pl][s], a[u][s], b[u][pl]);
    };
    if (n >= U) {
#pragma unroll
        for (int u = 0; u < U; ++u) fill(u, u);
        between();
        int i = 0;
        for (; i + 2 * U <= n; i += U) {               // every refill of such a trip is a k-block of the range
#pragma unroll
            for (int u = 0; u < U; ++u) { use(u); fill(u, i + u + U); }
        }
        const int extra = n - i - U;                   // 0 .. U-1 k-blocks still to request; the slots hold i .. i+U-1
#pragma unroll
        for (int u = 0; u < U; ++u) {
            use(u);
            if (u < extra) fill(u, i + u + U);
        }
#pragma unroll
        for (int u = 0; u + 1 < U; ++u)
            if (u < extra) use(u);
    } else {                                           // a K range shorter than the ring
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (u < n) fill(u, u);
        between();
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (u < n) use(u);
    }
}

// LDS of one workgroup's block function
template <class T, int EPI, int TN, int NW, bool PACK> struct GemmLds {
    static constexpr int NA = (EPI == EPI_GU) ? 2 * TN : TN;
    static constexpr int NPL = PACK ? 1 : T::NP;
    static constexpr bool kNormed = (EPI != EPI_RES);
    f32x4 red[NW][NPL][NA][64];
    float epi_a[(EPI == EPI_RES || EPI == EPI_LM) ? NA * 256 : 1];
    float epi_b[EPI == EPI_RES ? NA * 256 : 1];
    float fin_a[kNormed ? NW * 64 : 1];
    float fin_b[kNormed ? NW * 64 : 1];
    float rscale[16];
};

// One workgroup's share of the contraction: block bid owns tiles bid*TN .. bid*TN+TN-1.
//
// Two-plane (bf16) activations: the hi and the lo plane are contracted into separate sums, added once at the end.
// PACK (passes of at most 8 rows): both planes share one operand, rows in columns 0..7 hi and 8..15 lo, so a
// k-block costs one fragment load and one MFMA; otherwise each plane has its own operand and accumulators.  Either
// way an output element is (sum over waves of its hi sums) + (sum over waves of its lo sums): the same bits.
template <class T, int EPI, int TN, int NW, int U, bool PACK>
__device__ __forceinline__ void gemm_block(const GemmArgs& a, const int bid, GemmLds<T, EPI, TN, NW, PACK>& lds) {
    constexpr int NA = (EPI == EPI_GU) ? 2 * TN : TN;
    constexpr int NT = NW * 64;
    constexpr int NPL = PACK ? 1 : T::NP;               // operands (and accumulator sets) per k-block
    static_assert(!PACK || T::NP == 2, "packing is for two-plane activations");
    constexpr bool kNormed = (EPI != EPI_RES);          // input went through RMSNorm: needs the row scale
    auto& red = lds.red;
    auto& epi_a = lds.epi_a;
    auto& epi_b = lds.epi_b;
    auto& fin_a = lds.fin_a;
    auto& fin_b = lds.fin_b;
    auto& rscale = lds.rscale;

    // The wave index as a scalar: everything derived from it (this wave's K range, the trip counts of the stream) is
    // then scalar too and the stream's control flow is real branches.  As a vector value the conditions become lane
    // masks, and a short conditional block is then executed with an empty mask instead of being branched around;
    // the matrix-core instructions do not honour the mask.
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);

    int tile[NA];
    bool tval[NA];
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        tile[t] = bid * TN + t;
        tval[t] = tile[t] < a.n_tiles;
        if constexpr (EPI == EPI_GU) { tile[TN + t] = tile[t]; tval[TN + t] = tval[t]; }
    }

    const u32x4* A[NA];
#pragma unroll
    for (int s = 0; s < NA; ++s) {
        const u32x4* base = (EPI == EPI_GU && s >= TN) ? a.W2 : a.W;
        A[s] = base + (size_t)(tval[s] ? tile[s] : 0) * a.w_tile_stride * ASD_WAVE + lane;
    }
    // K split over the waves: contiguous slices, or interleaved (wave w takes k-blocks w, w+NW, ...)
    int k_first, k_step, k_n;
    if (a.k_interleave) { k_first = w; k_step = NW; k_n = (a.KB - w + NW - 1) / NW; }
    else { k_first = (int)((long)w * a.KB / NW); k_step = 1; k_n = (int)((long)(w + 1) * a.KB / NW) - k_first; }

    // Work whose loads should hide under the weight stream, run once the first U steps are in flight:
    // ||y||^2 per row from the producing kernel's partials (same order in every workgroup), and for the
    // residual epilogue this thread's residual inputs.
    float syy = 0.f, sxy = 0.f;
    constexpr int NE = (EPI == EPI_RES) ? (NA * 256 + NT - 1) / NT : 1;
    constexpr int PRE_P = 8;                          // partials per thread requested ahead (the rest, if any, after the stream)
    float xpre[NE], gpre[NE], py[kNormed ? PRE_P : 1], px[kNormed ? PRE_P : 1];
    // Only requests here, no use: the loads queue in order, and waiting for one of these would wait for every
    // weight fragment requested before it, i.e. empty the ring once at the start of every kernel.
    auto early = [&]() {
        if constexpr (kNormed) {
            constexpr int J = NT / 16;
            const int m = tid & 15, j = tid >> 4;
#pragma unroll
            for (int q = 0; q < PRE_P; ++q) {
                const int p = j + q * J;
                const bool on = m < a.M && p < a.P_in;
                const float* src = &a.part_in[((size_t)(on ? p : 0) * 16 + (on ? m : 0)) * 2];
                const float y = src[1], x = src[0];
                py[q] = on ? y : 0.f;
                px[q] = on ? x : 0.f;
            }
        }
        if constexpr (EPI == EPI_RES) {
#pragma unroll
            for (int q = 0; q < NE; ++q) {
                const int e = tid + q * NT, s = e >> 8, m = (e >> 4) & 15, nl = e & 15;
                xpre[q] = 0.f; gpre[q] = 0.f;
                if (e < NA * 256 && m < a.M && tval[s]) {
                    xpre[q] = a.xres[(size_t)m * a.d + tile[s] * 16 + nl];
                    gpre[q] = a.g_next[tile[s] * 16 + nl];
                }
            }
        }
    };
    // ||y||^2 (and x.y in workgroup 0) per row from the partials, in the same order in every workgroup
    auto sum_partials = [&]() {
        if constexpr (kNormed) {
            constexpr int J = NT / 16;
            const int m = tid & 15, j = tid >> 4;
            if (m < a.M) {
#pragma unroll
                for (int q = 0; q < PRE_P; ++q)
                    if (j + q * J < a.P_in) { syy += py[q]; if (bid == 0) sxy += px[q]; }
                for (int p = j + PRE_P * J; p < a.P_in; p += J) {
                    syy += a.part_in[((size_t)p * 16 + m) * 2 + 1];
                    if (bid == 0) sxy += a.part_in[((size_t)p * 16 + m) * 2];
                }
            }
        }
    };

    f32x4 acc[NPL][NA];
#pragma unroll
    for (int pl = 0; pl < NPL; ++pl)
#pragma unroll
        for (int s = 0; s < NA; ++s) acc[pl][s] = f32x4{0.f, 0.f, 0.f, 0.f};
    // this lane's activation fragments; a lane whose row is not in use reads row 0's (the epilogues never look at
    // the columns of unused rows)
    const u32x4* Xl;
    if constexpr (PACK) Xl = a.X + ((lane & 8) ? a.x_plane : 0) + (lane >> 4) * a.RS + ((lane & 7) < a.M ? (lane & 7) : 0);
    else Xl = a.X + (lane >> 4) * a.RS + ((lane & 15) < a.M ? (lane & 15) : 0);
    stream_mma<T, NA, NPL, U>(A, Xl, 4 * a.RS, a.x_plane, k_first, k_step, k_n, a.w_kb_stride, acc, early);
    sum_partials();

#pragma unroll
    for (int pl = 0; pl < NPL; ++pl)
#pragma unroll
        for (int s = 0; s < NA; ++s) red[w][pl][s][lane] = acc[pl][s];

    if constexpr (kNormed) {
        constexpr int J = NT / 16;
        fin_a[tid] = syy; fin_b[tid] = sxy;
        __syncthreads();
        if (tid < 16) {
            float yy = 0.f, xy = 0.f;
            for (int jj = 0; jj < J; ++jj) { yy += fin_a[jj * 16 + tid]; xy += fin_b[jj * 16 + tid]; }
            rscale[tid] = rsqrtf(yy * a.inv_d + a.eps);
            float c = 0.f;
            if (bid == 0 && tid < a.M) {
                if (a.fin_cos_rows) {            // the partials come from a residual-add kernel: finish its cosine
                    const float xx = a.ssq[tid];
                    c = xy * rsqrtf(fmaxf(xx, 1e-16f) * fmaxf(yy, 1e-16f));
                    c = fminf(1.f, fmaxf(-1.f, c));
                    a.fin_cos_rows[tid] = c;
                }
                a.ssq[tid] = yy;
            }
            fin_b[tid] = c;
        }
        __syncthreads();
        if (bid == 0 && a.fin_cos_rows && tid == 0) {
            double sum = 0.0;
            for (int r = 0; r < a.M; ++r) sum += (double)fin_b[r];
            *a.fin_cos_acc += sum;
        }
    } else {
        __syncthreads();
    }

    // element (row m, local feature nl) of tile s summed over the waves in wave order
    auto gather = [&](int s, int m, int nl) -> float {
        const int src = (nl >> 2) * 16 + m, r = nl & 3;
        float v = 0.f;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) v += red[ww][0][s][src][r];
        if constexpr (T::NP == 2) {                      // the lo plane's sums: columns m + 8 (packed) or the second set
            float lo = 0.f;
#pragma unroll
            for (int ww = 0; ww < NW; ++ww) lo += PACK ? red[ww][0][s][src + 8][r] : red[ww][NPL - 1][s][src][r];
            v += lo;
        }
        return v;
    };

    if constexpr (EPI == EPI_QKV) {
        // The fused QKV weight is tiled so that tile j of a head holds head dims 8j..8j+7 in rows 0..7 and
        // the same dims + h/2, their rotary partners, in rows 8..15.
        using E = typename T::elem;
        const int hpt = a.h / 16, hh = a.h / 2;
        for (int e = tid; e < TN * 128; e += NT) {
            const int s = e >> 7, m = (e >> 3) & 15, nl = e & 7;
            if (m >= a.M || !tval[s]) continue;
            const int head = tile[s] / hpt, j = tile[s] % hpt;
            const float rs = rscale[m];
            float v0 = gather(s, m, nl) * rs, v1 = gather(s, m, nl + 8) * rs;
            const int i = j * 8 + nl;
            const int pos = a.st->pos + a.pos_off + m;
            if (head < a.n_h + a.n_kv) {
                const float c = a.rope[((size_t)pos * hh + i) * 2], sn = a.rope[((size_t)pos * hh + i) * 2 + 1];
                const float o0 = v0 * c - v1 * sn, o1 = v1 * c + v0 * sn;
                v0 = o0; v1 = o1;
            }
            if (head < a.n_h) {
                E* q = (E*)a.q + (size_t)head * a.h * a.RS;
                store_act<T>(q, a.q_plane, a.RS, i, m, v0);
                store_act<T>(q, a.q_plane, a.RS, i + hh, m, v1);
            } else {
                const bool isk = head < a.n_h + a.n_kv;
                const int kvh = isk ? head - a.n_h : head - a.n_h - a.n_kv;
                const int PT = a.page_tokens, page = a.page_table[pos / PT], slot = pos % PT;
                E* base = (E*)a.kv + ((size_t)page * a.n_kv + kvh) * 2 * PT * a.h;
                if (isk) {                       // into the chunk's K fragments
                    *(base + kv_k_off<T>(slot, i, a.h)) = T::from_f32(v0);
                    *(base + kv_k_off<T>(slot, i + hh, a.h)) = T::from_f32(v1);
                } else {                         // into the chunk's V^T fragments
                    *(base + kv_v_off<T>(slot, i, a.h)) = T::from_f32(v0);
                    *(base + kv_v_off<T>(slot, i + hh, a.h)) = T::from_f32(v1);
                }
            }
        }
        return;
    }

    if constexpr (EPI == EPI_GU) {
        for (int e = tid; e < TN * 256; e += NT) {
            const int s = e >> 8, m = (e >> 4) & 15, nl = e & 15;
            if (m >= a.M || !tval[s]) continue;
            const float rs = rscale[m];
            const float g = gather(s, m, nl) * rs, u = gather(TN + s, m, nl) * rs;
            const float act = g / (1.f + __expf(-g)) * u;
            store_act<T>(a.hmid, a.hmid_plane, a.RS, tile[s] * 16 + nl, m, act);
        }
        return;
    }

    if constexpr (EPI == EPI_RES) {
#pragma unroll
        for (int q = 0; q < NE; ++q) {
            const int e = tid + q * NT, s = e >> 8, m = (e >> 4) & 15, nl = e & 15;
            if (e >= NA * 256) break;
            float pxy = 0.f, pyy = 0.f;
            if (m < a.M && tval[s]) {
                const int n = tile[s] * 16 + nl;
                const float x = xpre[q];
                const float y = x + gather(s, m, nl);
                a.xres[(size_t)m * a.d + n] = y;
                store_act<T>(a.xb, a.xb_plane, a.RS, n, m, y * gpre[q]);
                pxy = x * y; pyy = y * y;
            }
            epi_a[e] = pxy; epi_b[e] = pyy;
        }
        __syncthreads();
        if (tid < 16) {
            float sxy = 0.f, syy = 0.f;
            for (int s = 0; s < NA; ++s)
                for (int nl = 0; nl < 16; ++nl) { sxy += epi_a[s * 256 + tid * 16 + nl]; syy += epi_b[s * 256 + tid * 16 + nl]; }
            a.part[((size_t)bid * 16 + tid) * 2] = sxy;
            a.part[((size_t)bid * 16 + tid) * 2 + 1] = syy;
        }
    }

    if constexpr (EPI == EPI_LM) {
        for (int e = tid; e < NA * 256; e += NT) {
            const int s = e >> 8, m = (e >> 4) & 15, nl = e & 15;
            float lg = -INFINITY;
            if (m < a.M && tval[s]) {
                lg = gather(s, m, nl) * rscale[m];
                a.logits[(size_t)m * a.V + tile[s] * 16 + nl] = lg;
            }
            epi_a[e] = lg;
        }
        __syncthreads();
        if (tid < 16) {
            AmaxPart best{-INFINITY, 0x7fffffff, 0.f, 0.f};
            for (int s = 0; s < NA; ++s)
                for (int nl = 0; nl < 16; ++nl) {
                    const float v = epi_a[s * 256 + tid * 16 + nl];
                    if (v > best.v) { best.v = v; best.i = tile[s] * 16 + nl; }
                }
            float se = 0.f;
            if (best.v != -INFINITY)
                for (int s = 0; s < NA; ++s)
                    for (int nl = 0; nl < 16; ++nl) se += __expf(epi_a[s * 256 + tid * 16 + nl] - best.v);
            a.amax_part[(size_t)bid * 16 + tid].v = best.v;
            a.amax_part[(size_t)bid * 16 + tid].i = best.i;
            a.amax_part[(size_t)bid * 16 + tid].s = se;
        }
    }
}

template <class T, int EPI, int TN, int NW, int U, bool PACK>
// The leading scalar parameters repeat what a wave needs for its first weight and activation requests: built with
// kernel-argument preloading they arrive in SGPRs with the wave (14 dwords at most), while the argument structure is
// fetched from memory, which costs the first requests of every launch ~0.4 us (measured: every GEMM launch 0.4 us
// shorter).  packed = k_interleave | M << 8 | RS << 16.
__global__ __launch_bounds__(NW * 64) void gemm_kernel(const u32x4* W, const u32x4* X, int32_t w_tile_stride, int32_t w_kb_stride, int32_t n_tiles,
                                                        int32_t KB, int32_t packed, int32_t, int64_t x_plane, const u32x4* W2, const GemmArgs a) {
    GemmArgs b = a;
    b.W = W; b.W2 = W2; b.X = X; b.w_tile_stride = w_tile_stride; b.w_kb_stride = w_kb_stride; b.x_plane = x_plane;
    b.n_tiles = n_tiles; b.KB = KB; b.k_interleave = packed & 255; b.M = (packed >> 8) & 255; b.RS = packed >> 16;
    __shared__ GemmLds<T, EPI, TN, NW, PACK> lds;
    gemm_block<T, EPI, TN, NW, U, PACK>(b, blockIdx.x, lds);
}
