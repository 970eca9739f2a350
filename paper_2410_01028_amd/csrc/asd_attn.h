// Decode attention over the paged KV cache for up to 16 query rows (split-KV + fixed-order merge).
//
// Work item = (query head, chunk of 64 keys at absolute positions [64c, 64c+64)), one wave.
// Scores S[key][row] and the output O[dim][row] are both matrix-core products with the 16
// query rows as columns, so a row's result never depends on how many rows the call has;
// chunk boundaries are absolute, and the merge walks the chunks in ascending order.  A row
// at position p sees keys 0..p (causal among the rows of the call as well).
//
// Cache page layout per (page, kv head): K[page_tokens][h] then V transposed [h][page_tokens],
// which makes the fragments of both products contiguous 16-byte loads:
//   scores: A = K rows (keys x head-dim block), B = q (tiled [h/KE][16][KE]);
//   output: A = V^T rows (head dims x key block), B = P taken straight from the score
//   registers: a lane of group g holds, for its row, keys 4g..4g+3 of each 16-key score
//   tile; with the key order of the score tiles chosen per storage type below, those
//   registers are exactly the B fragment whose keys match a contiguous V^T load.
#pragma once
#include "asd_common.h"

struct AttnArgs {
    const void* q;            // [n_h][h/KE][16][KE]
    const void* kv;           // this layer's cache pages
    const int32_t* page_table;
    const DevState* st;
    int32_t pos_off, M;
    int32_t n_h, n_kv, h, page_tokens;
    int32_t nc_stride;        // chunks per head in the partial buffers
    float scale;              // 1/sqrt(h)
    float* o_part;            // [n_h][nc_stride][16][h] unnormalised partial outputs
    float2* ml_part;          // [n_h][nc_stride][16] (chunk max, chunk sum)
    void* out;                // tiled activation [n_h*h] (merge)
};

// key (0..63, relative to the chunk) held by score tile kt, tile row r
template <class T> __device__ __forceinline__ int score_key(int kt, int r);
template <> __device__ __forceinline__ int score_key<BF16>(int kt, int r) {
    return 32 * (kt >> 1) + 8 * (r >> 2) + 4 * (kt & 1) + (r & 3);    // two tiles interleave into one 32-key block
}
template <> __device__ __forceinline__ int score_key<F32>(int kt, int r) { return 16 * kt + r; }

template <class T, int H>
__global__ __launch_bounds__(64) void attn_partial_kernel(const AttnArgs a) {
    using E = typename T::elem;
    constexpr int KE = T::KE;
    constexpr int HS = H / (4 * KE);            // fragment steps over the head dimension
    constexpr int HT = H / 16;                  // output tiles over the head dimension
    constexpr int KST = 64 / (4 * KE);          // fragment steps over the 64 keys (2 bf16, 4 fp32)
    const int c = blockIdx.x, head = blockIdx.y, lane = threadIdx.x;
    const int g = lane >> 4, m = lane & 15, r = lane & 15;
    const int pos0 = a.st->pos + a.pos_off;
    if (c * ASD_CHUNK > pos0 + a.M - 1) return;          // no row of this call sees this chunk
    const int kvh = head / (a.n_h / a.n_kv);
    const int PT = a.page_tokens;
    const int page = a.page_table[(c * ASD_CHUNK) / PT], slot0 = (c * ASD_CHUNK) % PT;
    const E* Kp = (const E*)a.kv + ((size_t)page * a.n_kv + kvh) * 2 * PT * H;
    const E* Vp = Kp + (size_t)PT * H;
    const E* qp = (const E*)a.q + (size_t)head * H * ASD_ROWS;

    // ---- scores: 4 tiles of 16 keys
    u32x4 qf[HS];
#pragma unroll
    for (int hs = 0; hs < HS; ++hs) qf[hs] = *(const u32x4*)(qp + ((size_t)(hs * 4 + g) * ASD_ROWS + m) * KE);
    f32x4 s[4];
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
        s[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
        const E* krow = Kp + (size_t)(slot0 + score_key<T>(kt, r)) * H + g * KE;
#pragma unroll
        for (int hs = 0; hs < HS; ++hs) {
            const u32x4 kf = __builtin_nontemporal_load((const u32x4*)(krow + hs * 4 * KE));
            mma16<T>(s[kt], kf, qf[hs]);
        }
    }
    // ---- V^T fragments (independent of the scores: issue early)
    u32x4 vf[HT][KST];
#pragma unroll
    for (int ht = 0; ht < HT; ++ht)
#pragma unroll
        for (int ks = 0; ks < KST; ++ks)
            vf[ht][ks] = __builtin_nontemporal_load(
                (const u32x4*)(Vp + (size_t)(ht * 16 + r) * PT + slot0 + ks * 4 * KE + g * KE));

    // ---- causal mask, chunk max, exponentials, chunk sum (per row = per column m)
    const int row_pos = pos0 + m;
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int key = c * ASD_CHUNK + score_key<T>(kt, 4 * g + j);
            const float v = (key <= row_pos) ? s[kt][j] * a.scale : -INFINITY;
            s[kt][j] = v;
            mx = fmaxf(mx, v);
        }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    float l = 0.f;
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float p = (s[kt][j] == -INFINITY) ? 0.f : __expf(s[kt][j] - mx);
            p = T::to_f32(T::from_f32(p));          // the value the matrix cores will see
            s[kt][j] = p;
            l += p;
        }
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);

    // ---- output: O[dim][row] += V^T[dim][keys] * P[keys][row]
    u32x4 pf[KST];
    if constexpr (KE == 8) {
#pragma unroll
        for (int ks = 0; ks < KST; ++ks)
#pragma unroll
            for (int w2 = 0; w2 < 4; ++w2) {
                const f32x4& t = s[2 * ks + (w2 >> 1)];
                const uint32_t lo = BF16::from_f32(t[(w2 & 1) * 2]), hi = BF16::from_f32(t[(w2 & 1) * 2 + 1]);
                pf[ks][w2] = lo | (hi << 16);
            }
    } else {
#pragma unroll
        for (int ks = 0; ks < KST; ++ks)
#pragma unroll
            for (int j = 0; j < 4; ++j) pf[ks][j] = __float_as_uint(s[ks][j]);
    }
    float* op = a.o_part + (((size_t)head * a.nc_stride + c) * ASD_ROWS + m) * H;
#pragma unroll
    for (int ht = 0; ht < HT; ++ht) {
        f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KST; ++ks) mma16<T>(o, vf[ht][ks], pf[ks]);
        if (m < a.M) *(f32x4*)(op + ht * 16 + 4 * g) = o;
    }
    if (g == 0 && m < a.M) a.ml_part[((size_t)head * a.nc_stride + c) * ASD_ROWS + m] = float2{mx, l};
}

// Merge the chunk partials of one (head, row) in ascending chunk order and write the tiled activation.
template <class T, int H>
__global__ __launch_bounds__(H) void attn_merge_kernel(const AttnArgs a) {
    using E = typename T::elem;
    const int head = blockIdx.x, m = blockIdx.y, hd = threadIdx.x;
    const int pos = a.st->pos + a.pos_off + m;
    const int nc = pos / ASD_CHUNK + 1;
    const float2* ml = a.ml_part + (size_t)head * a.nc_stride * ASD_ROWS + m;
    float gmax = -INFINITY;
    for (int c = 0; c < nc; ++c) gmax = fmaxf(gmax, ml[(size_t)c * ASD_ROWS].x);
    float L = 0.f, o = 0.f;
    const float* op = a.o_part + ((size_t)head * a.nc_stride * ASD_ROWS + m) * H + hd;
    for (int c = 0; c < nc; ++c) {
        const float2 v = ml[(size_t)c * ASD_ROWS];
        const float w = __expf(v.x - gmax);
        L += v.y * w;
        o += op[(size_t)c * ASD_ROWS * H] * w;
    }
    ((E*)a.out)[act_index<T>(head * H + hd, m)] = T::from_f32(o / L);
}
