// Small kernels around the contractions: embedding gather, accept/rollback, decoding state,
// rotary table, weight re-tiling, the on-device synthetic weight generator, a plain copy.
#pragma once
#include "asd_common.h"

// ---------------------------------------------------------------- embedding + first norm statistics
// grid (EMBED_SPLIT, rows): x = E[token], the tiled copy x * gain for the first kept norm, and this
// workgroup's share of ||x||^2 as partial [split][16][2] (slot 1; slot 0 unused) for the next kernel.
#define EMBED_SPLIT 8
#define EMBED_THREADS 256
template <class T>
__device__ __forceinline__ void embed_block(const typename T::elem* E, const int32_t* tokens, int d, int vocab, DevState* st, const float* g_first,
                                            float* xres, void* xb, size_t xb_plane, int rs, float* part, const int sp, const int m, float* red) {
    using El = typename T::elem;
    const int tid = threadIdx.x, nt = EMBED_THREADS;
    // a token id that is not a row of the table (possible when the ids come from device memory the host never saw)
    // must not become an address: it reads row 0 and raises the state's error bit
    int tok = tokens[m];
    if ((unsigned)tok >= (unsigned)vocab) {
        tok = 0;
        if (tid == 0 && sp == 0) __hip_atomic_fetch_or(&st->err, (int)DEV_ERR_TOKEN, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const El* row = E + (size_t)tok * d;
    const int per = (d + EMBED_SPLIT - 1) / EMBED_SPLIT, lo = sp * per, hi = min(d, lo + per);
    float ss = 0.f;
    for (int i = lo + tid; i < hi; i += nt) {
        const float x = T::to_f32(row[i]);
        xres[(size_t)m * d + i] = x;
        store_act<T>(xb, xb_plane, rs, i, m, x * g_first[i]);
        ss += x * x;
    }
    red[tid] = ss;
    __syncthreads();
    for (int s = nt / 2; s > 0; s >>= 1) {
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    if (tid == 0) { part[((size_t)sp * 16 + m) * 2] = 0.f; part[((size_t)sp * 16 + m) * 2 + 1] = red[0]; }
    __syncthreads();
}
template <class T>
__global__ __launch_bounds__(EMBED_THREADS) void embed_kernel(const typename T::elem* E, const int32_t* tokens, int d, int vocab, DevState* st,
                                                    const float* g_first, float* xres, void* xb, size_t xb_plane, int rs, float* part) {
    __shared__ float red[EMBED_THREADS];
    embed_block<T>(E, tokens, d, vocab, st, g_first, xres, xb, xb_plane, rs, part, blockIdx.x, blockIdx.y, red);
}

// ---------------------------------------------------------------- decoding state
__global__ void set_state_kernel(DevState* st, int pos, int emitted, int target, int reset_counts, int index_base = 0) {
    st->pos = pos; st->emitted = emitted; st->target = target; st->index_base = index_base; st->err = 0;
    if (reset_counts) { st->cycles = 0; st->drafted = 0; st->accepted = 0; }
}
__global__ void set_token_kernel(int32_t* tokbuf, int32_t tok) { tokbuf[0] = tok; }

// After the LM head: pick each row's greedy token from the per-workgroup candidates (largest
// logit, lowest index on ties), then, by mode,
//   FIN_NONE    nothing more;
//   FIN_DRAFT   draft step j: the drafted token becomes row j+1 of the coming verification pass, and its
//               softmax probability goes to the decoding state (what an adaptive draft exit looks at);
//   FIN_ACCEPT  accept / rollback after a verification pass over rows [last, d_1..d_kk], g_i = the
//               full model's choice after row i: a = length of the longest prefix with
//               d_{i+1} == g_i; emit d_1..d_a, g_a; the cache keeps pos + a + 1 positions; g_a is
//               the next cycle's first row.
enum { FIN_NONE = 0, FIN_DRAFT = 1, FIN_ACCEPT = 2 };
struct AmaxCand { float v; int32_t i; float s; float pad; };
__device__ __forceinline__ bool amax_better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }
// one workgroup; wave w handles rows w, w + (waves), ...; candidates are [workgroup][16 rows]
__device__ __forceinline__ void finish_block(const AmaxCand* cand, int P, int M, int V, int32_t* argmax, int mode, int j_or_kk,
                                             DevState* st, int32_t* tokbuf, int32_t* out, int* win) {
    const int tid = threadIdx.x, lane = tid & 63, nw = blockDim.x >> 6;
    // what the accept step reads is requested now, so that it is there when the rows' winners are known
    int tb[16], st_emitted = 0, st_target = 0;
    if (tid == 0 && mode == FIN_ACCEPT) {
#pragma unroll
        for (int q = 0; q < 16; ++q) tb[q] = q <= j_or_kk ? tokbuf[q] : 0;
        st_emitted = st->emitted; st_target = st->target;
    }
    for (int m = tid >> 6; m < M; m += nw) {
        float v = -INFINITY; int idx = 0x7fffffff;
        // eight candidates per lane and trip, all requested before the first is looked at (one memory round trip per
        // trip instead of one per candidate); a lane past the end re-reads the last candidate, which changes nothing
        for (int p0 = lane; p0 < P; p0 += 64 * 8) {
            float cv[8]; int ci[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int p = p0 + 64 * u < P ? p0 + 64 * u : P - 1;
                cv[u] = cand[(size_t)p * 16 + m].v;
                ci[u] = cand[(size_t)p * 16 + m].i;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (amax_better(cv[u], ci[u], v, idx)) { v = cv[u]; idx = ci[u]; }
        }
        for (int o = 32; o > 0; o >>= 1) {
            const float ov = __shfl_xor(v, o); const int oi = __shfl_xor(idx, o);
            if (amax_better(ov, oi, v, idx)) { v = ov; idx = oi; }
        }
        // a row without a finite maximum (NaN weights) leaves no candidate: its token must still be a valid id,
        // because the next pass uses it as an address into the embedding table
        if ((unsigned)idx >= (unsigned)V) {
            idx = 0;
            if (lane == 0) __hip_atomic_fetch_or(&st->err, (int)DEV_ERR_LOGITS, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (lane == 0) { win[m] = idx; argmax[m] = idx; }
        if (mode == FIN_DRAFT && m == 0) {
            // confidence of the drafted token: 1 / sum_i exp(logit_i - max), from the per-workgroup sums
            float se = 0.f;
            for (int p0 = lane; p0 < P; p0 += 64 * 8) {          // ascending p per lane, as before; requests batched
                float cs[8], cv[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int p = p0 + 64 * u < P ? p0 + 64 * u : P - 1;
                    cs[u] = cand[(size_t)p * 16].s;
                    cv[u] = cand[(size_t)p * 16].v;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (p0 + 64 * u < P) se += cs[u] * __expf(cv[u] - v);
            }
            for (int o = 32; o > 0; o >>= 1) se += __shfl_xor(se, o);
            if (lane == 0) st->conf = 1.f / se;
        }
    }
    __syncthreads();
    if (tid != 0) return;
    if (mode == FIN_DRAFT) {
        tokbuf[j_or_kk + 1] = win[0];
    } else if (mode == FIN_ACCEPT) {
        const int kk = j_or_kk;
        int a = 0;
        while (a < kk && tb[a + 1] == win[a]) ++a;
        int e = st_emitted;
        for (int q = 1; q <= a && e < st_target; ++q) out[e++] = tb[q];
        if (e < st_target) out[e++] = win[a];
        st->emitted = e;
        st->pos += a + 1;
        st->cycles += 1; st->drafted += kk; st->accepted += a;
        tokbuf[0] = win[a];
    }
}
__global__ __launch_bounds__(1024) void finish_kernel(const AmaxCand* cand, int P, int M, int V, int32_t* argmax, int mode, int j_or_kk,
                                                      DevState* st, int32_t* tokbuf, int32_t* out) {
    __shared__ int win[16];
    finish_block(cand, P, M, V, argmax, mode, j_or_kk, st, tokbuf, out, win);
}

// ---------------------------------------------------------------- helpers of the entry point that allocates nothing
// clears n 32-bit words (counters and running sums that must start at zero; a kernel, not a memset, so that a caller
// may record the call into a HIP graph)
__global__ void zero_words_kernel(uint32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}
// one bit per sublayer of a skip mask, passed to a kernel by value
struct MaskBits { uint32_t w[128]; };
// mean over the rows of every sublayer's cosine (a removed sublayer reports exactly 1), to a caller's device buffer
__global__ void cos_mean_kernel(const double* cos_acc, int n_sub, int rows, MaskBits skip, float* out) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < n_sub) out[j] = ((skip.w[j >> 5] >> (j & 31)) & 1u) ? 1.f : (float)(cos_acc[j] / (double)rows);
}

// ---------------------------------------------------------------- rotary table: cos/sin(pos * theta^(-2i/h)) in double
__global__ void rope_table_kernel(float* tab, int max_seq, int half, double theta) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)max_seq * half) return;
    const int pos = (int)(idx / half), i = (int)(idx % half);
    const double ang = (double)pos * pow(theta, -(double)i / (double)half);
    tab[idx * 2] = (float)cos(ang);
    tab[idx * 2 + 1] = (float)sin(ang);
}

__global__ void iota_kernel(int32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = i;
}

// ---------------------------------------------------------------- weight tiling
// A tiled matrix is a set of 1 KiB fragments addressed by (tile, k-block): fragment index =
// (tile0 + tile) * ts + kb * ks with {ts, ks} = {KB, 1} (tile-major: a tile's K range is contiguous) or
// {1, total tiles} (k-major: the fragments of all tiles for one k-block are contiguous).  Inside a
// fragment lane 16g + r holds tile row r, k = kb*4KE + g*KE .. +KE.  rope_h != 0 selects the row order of
// the fused QKV matrix: tile j of a head holds head dims 8j..8j+7 in rows 0..7 and the same dims + h/2
// (their rotary partners) in rows 8..15.
struct TileMap {
    int64_t ts, ks;
    int32_t tile0, KB, rope_h;
};
__device__ __forceinline__ size_t tm_frag(const TileMap& tm, int tile, int kb) {
    return (size_t)(tm.tile0 + tile) * tm.ts + (size_t)kb * tm.ks;
}
__device__ __forceinline__ int tm_row(const TileMap& tm, int tile, int r) {
    if (!tm.rope_h) return tile * 16 + r;
    const int hpt = tm.rope_h / 16, head = tile / hpt, j = tile % hpt;
    return head * tm.rope_h + 8 * j + (r & 7) + (r >> 3) * (tm.rope_h / 2);
}
// f enumerates (tile, kb, lane) of one tensor; returns false when out of range
__device__ __forceinline__ bool tm_decode(const TileMap& tm, size_t f, int N, int* tile, int* kb, int* lane) {
    if (f >= (size_t)(N / 16) * tm.KB * 64) return false;
    *lane = (int)(f & 63);
    const size_t tk = f >> 6;
    *kb = (int)(tk % tm.KB); *tile = (int)(tk / tm.KB);
    return true;
}
template <class T>
__global__ void tile_weight_kernel(const typename T::elem* src, typename T::elem* dst, int N, int K, TileMap tm) {
    constexpr int KE = T::KE;
    int tile, kb, lane;
    if (!tm_decode(tm, (size_t)blockIdx.x * blockDim.x + threadIdx.x, N, &tile, &kb, &lane)) return;
    const int row = tm_row(tm, tile, lane & 15), k0 = kb * 4 * KE + (lane >> 4) * KE;
    typename T::elem* d = dst + (tm_frag(tm, tile, kb) * 64 + lane) * KE;
#pragma unroll
    for (int j = 0; j < KE; ++j) d[j] = (k0 + j < K) ? src[(size_t)row * K + k0 + j] : (typename T::elem)0;
}
template <class T>
__global__ void untile_weight_kernel(const typename T::elem* src, typename T::elem* dst, int N, int K, TileMap tm) {
    constexpr int KE = T::KE;
    int tile, kb, lane;
    if (!tm_decode(tm, (size_t)blockIdx.x * blockDim.x + threadIdx.x, N, &tile, &kb, &lane)) return;
    const int row = tm_row(tm, tile, lane & 15), k0 = kb * 4 * KE + (lane >> 4) * KE;
    const typename T::elem* sfr = src + (tm_frag(tm, tile, kb) * 64 + lane) * KE;
#pragma unroll
    for (int j = 0; j < KE; ++j) if (k0 + j < K) dst[(size_t)row * K + k0 + j] = sfr[j];
}

// ---------------------------------------------------------------- synthetic weights (counter based)
// Same recipe as the host input generator: element i of a tensor draws mix64(stream + (c+1)*GOLD)
// for c = 2i, 2i+1; the sum of the eight 16-bit fields minus 262140, times one fp32 constant,
// rounded once to the storage type.
__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27; z *= 0x94D049BB133111EBULL;
    z ^= z >> 31; return z;
}
__device__ __forceinline__ int field_sum(uint64_t r) {
    return (int)(r & 0xFFFF) + (int)((r >> 16) & 0xFFFF) + (int)((r >> 32) & 0xFFFF) + (int)(r >> 48);
}
__device__ __forceinline__ float synth_value(uint64_t stream, uint64_t i, float cst) {
    const uint64_t G = 0x9E3779B97F4A7C15ULL;
    const int s = field_sum(mix64(stream + (2 * i + 1) * G)) + field_sum(mix64(stream + (2 * i + 2) * G)) - 262140;
    return (float)s * cst;
}
// tiled == 0: dst row-major [N][K];  tiled != 0: dst in the tiled weight layout (K padded with zeros)
template <class T>
__global__ void synth_weight_kernel(typename T::elem* dst, int N, int K, TileMap tm, uint64_t stream, float cst, int tiled) {
    constexpr int KE = T::KE;
    const size_t f = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (tiled) {
        int tile, kb, lane;
        if (!tm_decode(tm, f, N, &tile, &kb, &lane)) return;
        const int row = tm_row(tm, tile, lane & 15), k0 = kb * 4 * KE + (lane >> 4) * KE;
        typename T::elem* d = dst + (tm_frag(tm, tile, kb) * 64 + lane) * KE;
#pragma unroll
        for (int j = 0; j < KE; ++j)
            d[j] = (k0 + j < K) ? T::from_f32(synth_value(stream, (uint64_t)row * K + k0 + j, cst)) : (typename T::elem)0;
    } else {
        if (f >= ((size_t)N * K + KE - 1) / KE) return;
#pragma unroll
        for (int j = 0; j < KE; ++j) {
            const size_t i = f * KE + j;
            if (i < (size_t)N * K) dst[i] = T::from_f32(synth_value(stream, i, cst));
        }
    }
}
__global__ void fill_f32_kernel(float* p, size_t n, float v) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// ---------------------------------------------------------------- plain copy (byte-counter calibration, achievable HBM rate)
__global__ __launch_bounds__(256) void copy_kernel(const u32x4* src, u32x4* dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}
