// Prompt processing as large-M contractions: the pass that fills the KV cache and measures the prompt's
// average cosine similarity per sublayer (Section 3.2, the definition of C_l) before the draft / verify loop starts.
//
// The prompt is processed in blocks of up to PF_ROWS rows, layer by layer, so every weight is read once per
// block instead of once per 16 rows.  Activations of a block are kept as 16-row chunks, each chunk in the same
// tiled layout the decode kernels use with a row stride of 16 ([K/KE][16][KE], hi and lo planes for bf16):
// one (chunk, k-block) fragment is one contiguous KiB that a wave loads with one instruction, and the decode
// attention kernel runs unchanged on a chunk.
//
// pf_gemm_kernel: a workgroup of NW waves owns NW*NA weight tiles (16 output features each) x NC chunks of
// rows and, with a K split, one slice of K.  Per k-block the waves stage the NC chunks' activation fragments
// in LDS (double buffered, one barrier per k-block); each wave streams its own NA weight fragments from
// global memory and feeds NA*NC accumulators.  Workgroups that share weights (same features, other rows)
// and those that share activations run at the same time on the same XCD, so both are served by its L2.
//   PF_QKV  RMSNorm scale, rotary embedding, q -> chunked q buffer, k/v -> paged cache
//   PF_GU   RMSNorm scale, silu(gate) * up -> chunked activation
//   PF_RAW  the slice's partial sums -> raw[k slice][row][feature]; pf_resid_kernel then adds the slices to
//           the residual stream in slice order, writes the normed copy for the next sublayer and finishes the
//           cosine tap of every row.
#pragma once
#include <type_traits>
#include "asd_gemm.h"

#define PF_ROWS 512                    // rows per prompt block
#define PF_CHUNKS (PF_ROWS / 16)
#define PF_MAX_KSPLIT 8

enum { PF_QKV = 0, PF_RAW = 1, PF_GU = 2 };

struct PfArgs {
    const u32x4 *W, *W2, *X;
    int64_t x_plane, x_chunk;        // fragment strides of X: between planes, between 16-row chunks
    int32_t n_tiles, KB;
    int64_t w_tile_stride, w_kb_stride;
    int32_t n_fb, n_rb, ksplit;      // feature blocks (NW*NA tiles each), row blocks (NC chunks each), K slices
    int32_t rows;                    // valid rows of this prompt block
    const float* rscale;             // [PF_ROWS] RMSNorm scale of each row (PF_QKV, PF_GU)
    float* raw;                      // PF_RAW: [ksplit][PF_ROWS][16 * n_tiles]
    // PF_QKV
    int32_t pos0;                    // cache position of row 0
    const float* rope;
    void* q; int64_t q_plane, q_chunk;         // element strides
    void* kv; const int32_t* page_table;
    int32_t n_h, n_kv, h, page_tokens;
    // PF_GU
    void* hmid; int64_t hmid_plane, hmid_chunk;
};

// four consecutive single-plane elements (cache rows)
template <class T> __device__ __forceinline__ void store_elem4(typename T::elem* p, const float (&v)[4]) {
    if constexpr (sizeof(typename T::elem) == 2) {
        const uint32_t a = T::from_f32(v[0]), b = T::from_f32(v[1]), c = T::from_f32(v[2]), d = T::from_f32(v[3]);
        *(uint2*)p = uint2{a | (b << 16), c | (d << 16)};
    } else {
        *(float4*)p = float4{v[0], v[1], v[2], v[3]};
    }
}

template <class T, int EPI, int NA, int NC, int NW, int PD>
__global__ __launch_bounds__(NW * 64, PD >= 2 ? 2 : 1) void pf_gemm_kernel(const PfArgs a) {
    using E = typename T::elem;
    constexpr int NP = T::NP;
    constexpr int NAT = (EPI == PF_GU) ? 2 * NA : NA;
    constexpr int XF = NC * NP;                       // activation fragments per k-block of this row block
    constexpr int XW = (XF + NW - 1) / NW;            // ... staged by each wave
    __shared__ u32x4 xs[2][XF][64];

    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6), g = lane >> 4, m = lane & 15;
    // workgroup -> (feature block, row block, K slice): consecutive workgroup ids go to the 8 XCDs in turn, so the
    // XCD is the low 3 bits; on one XCD the row blocks and K slices of a feature block follow each other.
    const int L = blockIdx.x, inner = a.n_rb * a.ksplit;
    const int fb = ((L >> 3) / inner) * 8 + (L & 7), in = (L >> 3) % inner, rb = in % a.n_rb, ks = in / a.n_rb;
    if (fb >= a.n_fb) return;
    const int chunk0 = rb * NC;

    int tile[NA];
    bool tval[NA];
#pragma unroll
    for (int s = 0; s < NA; ++s) { tile[s] = (fb * NW + w) * NA + s; tval[s] = tile[s] < a.n_tiles; }
    const u32x4* A[NAT];
#pragma unroll
    for (int s = 0; s < NAT; ++s) {
        const u32x4* base = (EPI == PF_GU && s >= NA) ? a.W2 : a.W;
        A[s] = base + (size_t)(tval[s % NA] ? tile[s % NA] : 0) * a.w_tile_stride * ASD_WAVE + lane;
    }
    const int kb0 = (int)((long)ks * a.KB / a.ksplit), kb1 = (int)((long)(ks + 1) * a.KB / a.ksplit);
    const u32x4* Xp[XW];
#pragma unroll
    for (int i = 0; i < XW; ++i) {
        const int f = w + NW * i, c = (f < XF ? f : 0) / NP, pl = (f < XF ? f : 0) % NP;
        Xp[i] = a.X + (size_t)pl * a.x_plane + (size_t)(chunk0 + c) * a.x_chunk + lane;
    }

    f32x4 acc[NAT][NC];
#pragma unroll
    for (int s = 0; s < NAT; ++s)
#pragma unroll
        for (int c = 0; c < NC; ++c) acc[s][c] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Weight and activation fragments are requested PD k-blocks ahead of their use (register ring).  Every trip of
    // the main loop issues the same loads whatever the k-block (past the end of the range the last k-block is asked
    // for again and never used): the wait counts the compiler derives are exact only when no path skips a load, and
    // one conditional request is enough to turn every wait into a full drain, which undoes the prefetch.
    u32x4 an[PD][NAT], xg[PD][XW];
    auto issue = [&](int slot, int kb) {
#pragma unroll
        for (int i = 0; i < XW; ++i)
            if (XF % NW == 0 || w + NW * i < XF) xg[slot][i] = Xp[i][(size_t)kb * ASD_WAVE];
#pragma unroll
        for (int s = 0; s < NAT; ++s) an[slot][s] = A[s][(size_t)kb * a.w_kb_stride * ASD_WAVE];
    };
    // One k-block from ring slot p.  The slot's next request goes out only after its products (straight into the
    // same registers): asked for any earlier, the old values would have to be copied aside and the new ones copied
    // back at the loop's end, which the compiler can only do after waiting for them, every trip.
    auto k_block = [&](const int p, const int kb, auto prefetch) {
        const int buf = (kb - kb0) & 1;
#pragma unroll
        for (int i = 0; i < XW; ++i)
            if (XF % NW == 0 || w + NW * i < XF) xs[buf][w + NW * i][lane] = xg[p][i];
        __syncthreads();
        // all LDS reads of the k-block are requested before its first MFMA: one LDS latency per k-block, not one per pair
        u32x4 b[NC][NP];
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int pl = 0; pl < NP; ++pl) b[c][pl] = xs[buf][c * NP + pl][lane];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int pl = 0; pl < NP; ++pl)
#pragma unroll
                for (int s = 0; s < NAT; ++s) mma16<T>(acc[s][c], an[p][s], b[c][pl]);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (decltype(prefetch)::value) issue(p, kb + PD < kb1 ? kb + PD : kb1 - 1);
    };
#pragma unroll
    for (int p = 0; p < PD; ++p) issue(p, kb0 + p < kb1 ? kb0 + p : kb1 - 1);
    const int n_full = (kb1 - kb0) / PD * PD;
    for (int kbb = kb0; kbb < kb0 + n_full; kbb += PD) {
#pragma unroll
        for (int p = 0; p < PD; ++p) k_block(p, kbb + p, std::true_type{});
    }
#pragma unroll
    for (int p = 0; p + 1 < PD; ++p)                    // the last, partial round: nothing further to request
        if (kb0 + n_full + p < kb1) k_block(p, kb0 + n_full + p, std::false_type{});

    // ---- epilogues, straight from the accumulators: lane 16g + m holds features 4g..4g+3 of each tile for row m
    int row[NC];
    bool rv[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) { row[c] = (chunk0 + c) * 16 + m; rv[c] = row[c] < a.rows; }

    if constexpr (EPI == PF_RAW) {
        const int N = a.n_tiles * 16;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            if (!rv[c]) continue;
            float* dst = a.raw + ((size_t)ks * PF_ROWS + row[c]) * N + 4 * g;
#pragma unroll
            for (int s = 0; s < NA; ++s)
                if (tval[s]) *(f32x4*)(dst + tile[s] * 16) = acc[s][c];
        }
    }

    if constexpr (EPI == PF_GU) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            if (!rv[c]) continue;
            const float rs = a.rscale[row[c]];
#pragma unroll
            for (int s = 0; s < NA; ++s) {
                if (!tval[s]) continue;
                float v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float gt = acc[s][c][j] * rs, up = acc[NA + s][c][j] * rs;
                    v[j] = gt / (1.f + __expf(-gt)) * up;
                }
                store_act4<T>(a.hmid, a.hmid_plane, (int64_t)(chunk0 + c) * a.hmid_chunk, tile[s] * 16 + 4 * g, m, v);
            }
        }
    }

    if constexpr (EPI == PF_QKV) {
        // tile j of a head: rows 0..7 = head dims 8j..8j+7, rows 8..15 = the same dims + h/2 (rotary partners):
        // lane groups 0,1 hold the first halves, groups 2,3 their partners, 32 lanes away
        const int hpt = a.h / 16, hh = a.h / 2;
#pragma unroll
        for (int s = 0; s < NA; ++s) {
            if (!tval[s]) continue;                   // wave-uniform
            const int head = tile[s] / hpt, jt = tile[s] % hpt;
            const int i0 = jt * 8 + 4 * (g & 1), dim = i0 + (g >= 2 ? hh : 0);
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const float rs = rv[c] ? a.rscale[row[c]] : 0.f;
                float own[4], oth[4], v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) { own[j] = acc[s][c][j] * rs; oth[j] = __shfl_xor(own[j], 32); }
                if (!rv[c]) continue;
                const int pos = a.pos0 + row[c];
                if (head < a.n_h + a.n_kv) {
                    const float* rp = a.rope + ((size_t)pos * hh + i0) * 2;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float cs = rp[2 * j], sn = rp[2 * j + 1];
                        v[j] = g < 2 ? own[j] * cs - oth[j] * sn : own[j] * cs + oth[j] * sn;
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) v[j] = own[j];
                }
                if (head < a.n_h) {
                    store_act4<T>(a.q, a.q_plane, (int64_t)(chunk0 + c) * a.q_chunk, head * a.h + dim, m, v);
                } else {
                    const bool isk = head < a.n_h + a.n_kv;
                    const int kvh = isk ? head - a.n_h : head - a.n_h - a.n_kv;
                    const int PT = a.page_tokens, page = a.page_table[pos / PT], slot = pos % PT;
                    E* base = (E*)a.kv + ((size_t)page * a.n_kv + kvh) * 2 * PT * a.h;
                    if (isk) {                   // dim is a multiple of 4: the four values stay inside one lane's KE elements
                        store_elem4<T>(base + kv_k_off<T>(slot, dim, a.h), v);
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) base[kv_v_off<T>(slot, dim + j, a.h)] = T::from_f32(v[j]);
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------- rows of a block: embedding, residual add + cosine tap
// fixed-order sum of one value per thread (blockDim.x a power of two <= 256); result valid in thread 0
__device__ __forceinline__ float pf_block_sum(float v, float* red) {
    const int tid = threadIdx.x;
    red[tid] = v;
    __syncthreads();
    for (int s = blockDim.x / 2; s > 0; s >>= 1) {
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    const float r = red[0];
    __syncthreads();
    return r;
}

// grid = chunk-padded rows; rows at or beyond `rows` are zero-filled
template <class T>
__global__ __launch_bounds__(256) void pf_embed_kernel(const typename T::elem* E, const int32_t* tokens, int rows, int d, const float* g_first,
                                                       float* xres, void* xb, int64_t xb_plane, int64_t xb_chunk, float* ssq, float* rscale,
                                                       float inv_d, float eps) {
    __shared__ float red[256];
    const int r = blockIdx.x, tid = threadIdx.x;
    const bool valid = r < rows;
    const typename T::elem* src = E + (size_t)(valid ? tokens[r] : 0) * d;
    float ss = 0.f;
    for (int n0 = tid * 4; n0 < d; n0 += 1024) {
        float x[4], v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            x[j] = valid ? T::to_f32(src[n0 + j]) : 0.f;
            v[j] = x[j] * g_first[n0 + j];
            ss += x[j] * x[j];
        }
        *(float4*)&xres[(size_t)r * d + n0] = float4{x[0], x[1], x[2], x[3]};
        store_act4<T>(xb, xb_plane, (int64_t)(r / 16) * xb_chunk, n0, r % 16, v);
    }
    const float tot = pf_block_sum(ss, red);
    if (tid == 0) { ssq[r] = tot; rscale[r] = rsqrtf(tot * inv_d + eps); }
}

// grid = valid rows: y = x + sum of the K slices (slice order), residual stream, normed copy for the next sublayer,
// the row's cosine(x, y) (the summand of C_l, Section 3.2) and the statistics of y
template <class T>
__global__ __launch_bounds__(256) void pf_resid_kernel(const float* raw, int ksplit, int d, float* xres, void* xb, int64_t xb_plane,
                                                       int64_t xb_chunk, const float* g_next, float* ssq, float* rscale, float* cos_row,
                                                       float inv_d, float eps) {
    __shared__ float red[256];
    const int r = blockIdx.x, tid = threadIdx.x;
    float sxy = 0.f, syy = 0.f;
    // four 4-element pieces per thread and trip, every load of a trip requested before the first use: with two
    // workgroups per compute unit there is little else to hide the latency of a piece-by-piece walk
    constexpr int PB = 4;
    for (int base = tid * 4; base < d; base += PB * 1024) {
        float4 x4[PB], s4[PB], gn[PB], t4[PB][PF_MAX_KSPLIT - 1];
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            const int n0 = base + q * 1024;
            if (n0 < d) {
                x4[q] = *(const float4*)&xres[(size_t)r * d + n0];
                s4[q] = *(const float4*)&raw[(size_t)r * d + n0];
                gn[q] = *(const float4*)&g_next[n0];
#pragma unroll
                for (int k = 1; k < PF_MAX_KSPLIT; ++k)
                    if (k < ksplit) t4[q][k - 1] = *(const float4*)&raw[((size_t)k * PF_ROWS + r) * d + n0];
            }
        }
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            const int n0 = base + q * 1024;
            if (n0 < d) {
#pragma unroll
                for (int k = 1; k < PF_MAX_KSPLIT; ++k)
                    if (k < ksplit) { s4[q].x += t4[q][k - 1].x; s4[q].y += t4[q][k - 1].y; s4[q].z += t4[q][k - 1].z; s4[q].w += t4[q][k - 1].w; }
                const float x[4] = {x4[q].x, x4[q].y, x4[q].z, x4[q].w}, sv[4] = {s4[q].x, s4[q].y, s4[q].z, s4[q].w};
                const float gg[4] = {gn[q].x, gn[q].y, gn[q].z, gn[q].w};
                float y[4], v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) { y[j] = x[j] + sv[j]; v[j] = y[j] * gg[j]; sxy += x[j] * y[j]; syy += y[j] * y[j]; }
                *(float4*)&xres[(size_t)r * d + n0] = float4{y[0], y[1], y[2], y[3]};
                store_act4<T>(xb, xb_plane, (int64_t)(r / 16) * xb_chunk, n0, r % 16, v);
            }
        }
    }
    const float xy = pf_block_sum(sxy, red);
    const float yy = pf_block_sum(syy, red);
    if (tid == 0) {
        const float xx = ssq[r];
        float c = xy * rsqrtf(fmaxf(xx, 1e-16f) * fmaxf(yy, 1e-16f));
        c = fminf(1.f, fmaxf(-1.f, c));
        cos_row[r] = c;
        ssq[r] = yy;
        rscale[r] = rsqrtf(yy * inv_d + eps);
    }
}

// grid = sublayers: adds the block's rows' cosines (fixed order, double) to the running sums of C_l (Section 3.2)
__global__ __launch_bounds__(256) void pf_cos_sum_kernel(const float* cos_rows /* [sublayers][PF_ROWS] */, int rows, double* cos_acc) {
    __shared__ double red[256];
    const int j = blockIdx.x, tid = threadIdx.x;
    double s = 0.0;
    for (int r = tid; r < rows; r += 256) s += (double)cos_rows[(size_t)j * PF_ROWS + r];
    red[tid] = s;
    __syncthreads();
    for (int st = 128; st > 0; st >>= 1) {
        if (tid < st) red[tid] += red[tid + st];
        __syncthreads();
    }
    if (tid == 0) cos_acc[j] += red[0];
}

// one workgroup: hand row r of the block to the single-row decode buffers (residual, normed copy under the final
// norm's gain, ||x||^2 as the one partial the LM-head kernel sums), so that the LM head runs on it as row 0
template <class T>
__global__ __launch_bounds__(256) void pf_tail_kernel(const float* xres_pf, const float* ssq_pf, int r, int d, const float* g_final,
                                                      float* xres, void* xb, int64_t xb_plane, float* part) {
    for (int i = threadIdx.x; i < d; i += 256) {
        const float y = xres_pf[(size_t)r * d + i];
        xres[i] = y;
        store_act<T>(xb, (size_t)xb_plane, 1, i, 0, y * g_final[i]);
    }
    if (threadIdx.x == 0) { part[0] = 0.f; part[1] = ssq_pf[r]; }
}
