// Decode attention over the paged KV cache for up to 16 query rows (split-KV + fixed-order merges).
//
// A wave handles one chunk of 64 keys at absolute positions [64c, 64c+64) of one query head; scores
// S[key][row] and the output O[dim][row] are both matrix-core products with the 16 query rows as
// columns, so a row's result never depends on how many rows the call has.  Four waves (a group of
// 4 consecutive chunks = 256 keys, again at absolute positions) merge their results through LDS in
// ascending chunk order; the groups of a head spread over many compute units (one unit alone cannot
// pull a head's K/V fast enough).  When the context spans several groups, each group's partial goes to
// global memory and the groups are merged in ascending order by the group that arrives last (its four waves
// share the rows).  Partials and the arrival counter are
// exchanged with device-scope relaxed atomic stores / loads (served past the non-coherent per-XCD
// L2), ordered by waiting for the stores to complete before the counter is bumped; no cache-wide fence.
// A row at position p sees keys 0..p (causal among the rows of the call as well).
//
// Cache block per (page, kv head): per 64-key chunk the K fragments, then the V^T fragments, each fragment the
// contiguous 1 KiB register image of one load instruction (offsets: kv_k_frag_off / kv_v_frag_off):
//   scores: A = K rows (keys x head-dim block), B = q (tiled [h/KE][16][KE]);
//   output: A = V^T rows (head dims x key block), B = P taken straight from the score
//   registers: a lane of group g holds, for its row, keys 4g..4g+3 of each 16-key score
//   tile; with the key order of the score tiles chosen per storage type below, those
//   registers are exactly the B fragment whose keys match a contiguous V^T load.
#pragma once
#include "asd_common.h"
#include <type_traits>

#define ATT_GW 4                           // waves (chunks) per group
#define ATT_GROUP (ATT_GW * ASD_CHUNK)     // keys per group
#define ATT_RH 8                           // columns per LDS merge pass (one pass for the passes of at most 8 rows)
#define ATT_RB 2                           // (head, row) pairs a wave merges per round when it has more than one
#define ATT_CB 16                          // group partials requested up front per pair, ATT_RB pairs per round
#define ATT_CB1 36                         // the same with one pair per round (long contexts: one round trip up to 9216 keys)
#define ATT_NCL 4                          // group statistics per lane: up to 256 groups (64K positions) per head

// device-scope coherent scalar accesses (relaxed atomics: served past the per-XCD L2)
__device__ __forceinline__ void coherent_store2(float* p, float x, float y) {     // p 8-byte aligned
    __hip_atomic_store((uint64_t*)p, (uint64_t)__float_as_uint(x) | ((uint64_t)__float_as_uint(y) << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float coherent_load(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 coherent_load2(const float* p) {          // p 8-byte aligned
    const uint64_t u = __hip_atomic_load((const uint64_t*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return float2{__uint_as_float((uint32_t)u), __uint_as_float((uint32_t)(u >> 32))};
}

struct AttnArgs {
    const void* q;            // [n_h][h/KE][RS][KE], T::NP planes q_plane elements apart
    int64_t q_plane, out_plane;
    const void* kv;           // this layer's cache pages
    const int32_t* page_table;
    const DevState* st;
    int32_t pos_off, M, RS;   // rows in use, row stride of the activation buffers
    int32_t n_h, n_kv, h, page_tokens;
    int32_t nc_stride;        // groups per head in the partial buffers
    int32_t grid_groups;      // groups per head the launch covers (per-step kernels: see attn_unit)
    int32_t gh;               // query heads of one KV head a workgroup handles at once (a power of two, gh * RS <= 16)
    int32_t cap_chunks;       // 64-key chunks the cache has room for (the page table covers them all)
    float scale;              // 1/sqrt(h)
    float* o_part;            // [n_h][nc_stride][16][h] unnormalised group outputs
    float* ml_part;           // [n_h][nc_stride][16][2] (group max, group sum)
    unsigned* arrivals;       // [n_h] groups finished per head (returns to 0)
    void* out;                // tiled activation [n_h*h]
};

// Merge the group partials of RB (head, row) pairs, in ascending chunk order, and write the normalised output.
// Pair p of the n_pairs pairs of a workgroup's heads is head head0 + p / M, row p % M; this call takes pairs
// p0 .. p0 + RB - 1.  Chunk statistics with one chunk per lane, outputs with two head dims per lane; all
// loads of a round are requested before any is used.  One wave.  RB pairs per call with CB partials each requested
// up front; the sums run in ascending group order whatever RB and CB are, so the result is the same bits.
template <class T, int H, int RB = ATT_RB, int CB = ATT_CB>
__device__ __forceinline__ void attn_merge_rows(const AttnArgs& a, int head0, int p0, int n_pairs, int pos0, int lane) {
    const bool mine = 2 * lane < H;
    {
        float2 st[RB][ATT_NCL], v[RB][CB];
        int nc[RB], hd[RB], row[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int pp = p0 + rb < n_pairs ? p0 + rb : p0;        // an inactive slot aliases the first pair and loads nothing
            hd[rb] = head0 + pp / a.M; row[rb] = pp % a.M;
            const int head = hd[rb], mm = row[rb];
            nc[rb] = p0 + rb < n_pairs ? (pos0 + mm) / ATT_GROUP + 1 : 0;
            const float* ml = a.ml_part + ((size_t)head * a.nc_stride * ASD_ROWS + mm) * 2;
            const float* opm = a.o_part + ((size_t)head * a.nc_stride * ASD_ROWS + mm) * H + 2 * lane;
#pragma unroll
            for (int q = 0; q < ATT_NCL; ++q) {
                const int cc = lane + 64 * q;
                st[rb][q] = cc < nc[rb] ? coherent_load2(ml + (size_t)cc * ASD_ROWS * 2) : float2{-INFINITY, 0.f};
            }
#pragma unroll
            for (int u = 0; u < CB; ++u)
                v[rb][u] = (mine && u < nc[rb]) ? coherent_load2(opm + (size_t)u * ASD_ROWS * H) : float2{0.f, 0.f};
        }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            if (p0 + rb >= n_pairs) break;
            const int head = hd[rb], mm = row[rb];
            float gmax = -INFINITY;
#pragma unroll
            for (int q = 0; q < ATT_NCL; ++q) gmax = fmaxf(gmax, st[rb][q].x);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) gmax = fmaxf(gmax, __shfl_xor(gmax, o));
            float wq[ATT_NCL], L = 0.f;
#pragma unroll
            for (int q = 0; q < ATT_NCL; ++q) { wq[q] = __expf(st[rb][q].x - gmax); L += st[rb][q].y * wq[q]; }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) L += __shfl_xor(L, o);
            auto weight = [&](int cc) {
                float wgt = 0.f;
#pragma unroll
                for (int q = 0; q < ATT_NCL; ++q) { const float t = __shfl(wq[q], cc & 63); if ((cc >> 6) == q) wgt = t; }
                return wgt;
            };
            float2 acc = float2{0.f, 0.f};
#pragma unroll
            for (int u = 0; u < CB; ++u) {                 // ascending chunk order
                const float wgt = weight(u);
                if (u < nc[rb]) { acc.x += v[rb][u].x * wgt; acc.y += v[rb][u].y * wgt; }
            }
            const float* opm = a.o_part + ((size_t)head * a.nc_stride * ASD_ROWS + mm) * H + 2 * lane;
            for (int c0 = CB; c0 < nc[rb]; c0 += 8) {          // contexts beyond CB groups: 8 more per trip
                float2 x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    x[u] = (mine && c0 + u < nc[rb]) ? coherent_load2(opm + (size_t)(c0 + u) * ASD_ROWS * H) : float2{0.f, 0.f};
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const float wgt = weight(c0 + u);
                    if (c0 + u < nc[rb]) { acc.x += x[u].x * wgt; acc.y += x[u].y * wgt; }
                }
            }
            if (mine) {
                store_act<T>(a.out, a.out_plane, a.RS, head * H + 2 * lane, mm, acc.x / L);
                store_act<T>(a.out, a.out_plane, a.RS, head * H + 2 * lane + 1, mm, acc.y / L);
            }
        }
    }
}

// ---- pieces of one chunk's work, shared by the kernels below
// causal mask, chunk max, exponentials, chunk sum of one column (lane group g holds keys 4g..4g+3 of each score tile)
template <class T>
__device__ __forceinline__ void att_softmax(f32x4 (&s)[4], int c, int row_pos, float scale, int g, float& mx, float& l) {
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int key = c * ASD_CHUNK + score_key<T>(kt, 4 * g + j);
            const float v = (key <= row_pos) ? s[kt][j] * scale : -INFINITY;
            s[kt][j] = v;
            mx = fmaxf(mx, v);
        }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float p = (s[kt][j] == -INFINITY) ? 0.f : __expf(s[kt][j] - mx);
            s[kt][j] = p;
            l += p;
        }
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
}
// the probabilities as B fragments of the output product (hi + lo planes for bf16)
template <class T>
__device__ __forceinline__ void att_pfrags(const f32x4 (&s)[4], u32x4 (&pf)[64 / (4 * T::KE)][T::NP]) {
    constexpr int KE = T::KE, KST = 64 / (4 * KE), NP = T::NP;
    if constexpr (KE == 8) {
#pragma unroll
        for (int ks = 0; ks < KST; ++ks)
#pragma unroll
            for (int w2 = 0; w2 < 4; ++w2) {
                const f32x4& t = s[2 * ks + (w2 >> 1)];
                const float p0 = t[(w2 & 1) * 2], p1 = t[(w2 & 1) * 2 + 1];
                const uint32_t h0 = BF16::from_f32(p0), h1 = BF16::from_f32(p1);
                const uint32_t l0 = BF16::from_f32(p0 - BF16::to_f32((uint16_t)h0)), l1 = BF16::from_f32(p1 - BF16::to_f32((uint16_t)h1));
                pf[ks][0][w2] = h0 | (h1 << 16);
                if constexpr (NP == 2) pf[ks][1][w2] = l0 | (l1 << 16);
            }
    } else {
#pragma unroll
        for (int ks = 0; ks < KST; ++ks)
#pragma unroll
            for (int j = 0; j < 4; ++j) pf[ks][0][j] = __float_as_uint(s[ks][j]);
    }
}
// Merge a group's chunks through LDS, ATT_RH columns per pass, ascending chunk order; the result goes to the output
// (a context of one group) or to the group's partial.  Synchronises the workgroup; the chunk statistics are in sml.
template <class T, int H>
__device__ __forceinline__ void att_group_merge(const AttnArgs& a, int grp, int head, bool valid, int n_groups, int n_cols, int hw, int lane,
                                                const f32x4 (&o)[H / 16], float* so, const float* sml) {
    constexpr int HT = H / 16;
    const int g = lane >> 4, m = lane & 15;
    for (int m0 = 0; m0 < n_cols; m0 += ATT_RH) {
        if (m >= m0 && m < m0 + ATT_RH) {
#pragma unroll
            for (int ht = 0; ht < HT; ++ht) *(f32x4*)&so[((size_t)hw * ATT_RH + (m - m0)) * H + ht * 16 + 4 * g] = o[ht];
        }
        __syncthreads();
        const int n_here = n_cols - m0 < ATT_RH ? n_cols - m0 : ATT_RH;                 // columns of this pass
        for (int idx = hw * 64 + lane; idx < n_here * (H / 2); idx += ATT_GW * 64) {       // two head dims per thread and trip
            const int rr = idx / (H / 2), hd = 2 * (idx % (H / 2)), col = m0 + rr, mm = col % a.RS, hh = head + col / a.RS;
            if (!valid || col >= n_cols || mm >= a.M) continue;
            float gmax = -INFINITY;
#pragma unroll
            for (int ww = 0; ww < ATT_GW; ++ww) gmax = fmaxf(gmax, sml[(ww * ASD_ROWS + col) * 2]);
            float L = 0.f, acc0 = 0.f, acc1 = 0.f;
            if (gmax != -INFINITY) {
#pragma unroll
                for (int ww = 0; ww < ATT_GW; ++ww) {          // a chunk the row does not see has max -inf: weight 0
                    const float wgt = __expf(sml[(ww * ASD_ROWS + col) * 2] - gmax);
                    const float2 v = *(const float2*)&so[((size_t)ww * ATT_RH + rr) * H + hd];
                    L += sml[(ww * ASD_ROWS + col) * 2 + 1] * wgt;
                    acc0 += v.x * wgt;
                    acc1 += v.y * wgt;
                }
            }
            if (n_groups == 1) {
                store_act<T>(a.out, a.out_plane, a.RS, hh * H + hd, mm, acc0 / L);
                store_act<T>(a.out, a.out_plane, a.RS, hh * H + hd + 1, mm, acc1 / L);
            } else {
                const size_t row = ((size_t)hh * a.nc_stride + grp) * ASD_ROWS + mm;
                coherent_store2(a.o_part + row * H + hd, acc0, acc1);
                if (hd == 0) coherent_store2(a.ml_part + row * 2, gmax, L);
            }
        }
        __syncthreads();
    }
}

// One group (ATT_GW waves) of a.gh consecutive query heads that share a KV head, first head `head`: the 16 columns of
// the matrix-core products are (head, row) pairs, column j * RS + row for the j-th head (a.gh = 1: the rows of one
// head).  A column's arithmetic does not depend on what the other columns hold, so the result is the same bits for
// every gh.  Every thread of the calling workgroup must call this the same
// number of times (it synchronises the workgroup); `valid` = false makes the group a no-op, hw is the wave's
// index inside its group.  so: [ATT_GW][ATT_RH][H] floats, sml: [ATT_GW][16][2] floats, s_old: 1 word, per group.
template <class T, int H, bool EARLY = false>
__device__ __forceinline__ void attn_group(const AttnArgs& a, const int grp, const int head, const bool valid, const int hw,
                                           const int lane, float* so, float* sml, unsigned* s_old) {
    using E = typename T::elem;
    constexpr int KE = T::KE;
    constexpr int HS = H / (4 * KE);            // fragment steps over the head dimension
    constexpr int HT = H / 16;                  // output tiles over the head dimension
    constexpr int KST = 64 / (4 * KE);          // fragment steps over the 64 keys (2 bf16, 4 fp32)
    constexpr int NP = T::NP;
    const int g = lane >> 4, m = lane & 15, r = lane & 15;
    const int cj = m / a.RS, cm = m % a.RS;                 // this lane's column: head head + cj, row cm
    const bool col_ok = cj < a.gh && cm < a.M;
    const int n_cols = (a.gh - 1) * a.RS + a.M;             // columns in use: 0 .. n_cols-1 (those with cm >= M are holes)
    const int c = grp * ATT_GW + hw;
    const int kvh = head / (a.n_h / a.n_kv);
    const int PT = a.page_tokens;
    u32x4 qf[HS][NP], kf[4][HS], vf[HT][KST];
    auto request = [&]() {                  // this chunk's K and V^T fragments and the query fragments
        const int page = a.page_table[(c * ASD_CHUNK) / PT], slot0 = (c * ASD_CHUNK) % PT;
        const E* Cp = (const E*)a.kv + ((size_t)page * a.n_kv + kvh) * 2 * PT * H + kv_chunk_off<T>(slot0 / ASD_CHUNK, H) + lane * KE;
        const E* qp = (const E*)a.q + (size_t)(head + (col_ok ? cj : 0)) * H * a.RS;
#pragma unroll
        for (int hs = 0; hs < HS; ++hs)
#pragma unroll
            for (int pl = 0; pl < NP; ++pl)
                qf[hs][pl] = col_ok ? *(const u32x4*)(qp + pl * a.q_plane + ((size_t)(hs * 4 + g) * a.RS + cm) * KE)
                                    : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int hs = 0; hs < HS; ++hs)
                kf[kt][hs] = __builtin_nontemporal_load((const u32x4*)(Cp + kv_k_frag_off<T>(kt, hs, H)));
#pragma unroll
        for (int ht = 0; ht < HT; ++ht)
#pragma unroll
            for (int ks = 0; ks < KST; ++ks)
                vf[ht][ks] = __builtin_nontemporal_load((const u32x4*)(Cp + kv_v_frag_off<T>(ht, ks, H)));
    };
    // EARLY: the requests go out before the pass's position is known (the chunk exists in the cache whatever the
    // position; a chunk beyond the position is then dropped unused), which takes the position's load and the
    // comparison out of the chain position -> page -> fragments.
    if constexpr (EARLY) { if (valid && c < a.cap_chunks) request(); }
    const int pos0 = a.st->pos + a.pos_off, last = pos0 + a.M - 1;
    const int n_groups = last / ATT_GROUP + 1;
    const bool live = valid && grp * ATT_GROUP <= last;     // a group no row of the call sees is a no-op
    const bool active = live && c * ASD_CHUNK <= last;

    f32x4 o[HT];
#pragma unroll
    for (int ht = 0; ht < HT; ++ht) o[ht] = f32x4{0.f, 0.f, 0.f, 0.f};
    float mx = -INFINITY, l = 0.f;
    if (active) {
        if constexpr (!EARLY) request();
        // ---- scores: 4 tiles of 16 keys
        f32x4 s[4];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
            s[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int hs = 0; hs < HS; ++hs)
#pragma unroll
                for (int pl = 0; pl < NP; ++pl) mma16<T>(s[kt], kf[kt][hs], qf[hs][pl]);
        }

        // ---- causal mask, chunk max, exponentials, chunk sum (per column)
        att_softmax<T>(s, c, pos0 + cm, a.scale, g, mx, l);

        // ---- output: O[dim][row] += V^T[dim][keys] * P[keys][row]; P goes in as hi + lo planes for bf16
        u32x4 pf[KST][NP];
        att_pfrags<T>(s, pf);
#pragma unroll
        for (int ht = 0; ht < HT; ++ht)
#pragma unroll
            for (int ks = 0; ks < KST; ++ks)
#pragma unroll
                for (int pl = 0; pl < NP; ++pl) mma16<T>(o[ht], vf[ht][ks], pf[ks][pl]);
    }
    if (g == 0) { sml[(hw * ASD_ROWS + m) * 2] = mx; sml[(hw * ASD_ROWS + m) * 2 + 1] = l; }

    att_group_merge<T, H>(a, grp, head, live, n_groups, n_cols, hw, lane, o, so, sml);
    if (n_groups == 1) return;

    // ---- arrival: the group that completes the head's last outstanding group merges the groups
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);                   // this wave's partial stores have completed
    __syncthreads();
    if (hw == 0 && lane == 0) {
        *s_old = live ? __hip_atomic_fetch_add(a.arrivals + head, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0xffffffffu;
    }
    __syncthreads();
    if ((int)*s_old == n_groups - 1) {                // the group's waves share the (head, row) pairs, ATT_RB per wave and trip
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        if (hw == 0 && lane == 0) __hip_atomic_store(a.arrivals + head, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int n_pairs = a.gh * a.M;
        // One pair per call with ATT_CB1 partials requested up front, or ATT_RB pairs per call with ATT_CB each: whichever
        // takes the busiest wave through fewer memory round trips (the same sums in the same order either way)
        const int per_wave = (n_pairs + ATT_GW - 1) / ATT_GW;
        const int trips1 = per_wave * (1 + (n_groups > ATT_CB1 ? (n_groups - ATT_CB1 + 7) / 8 : 0));
        const int trips2 = (per_wave + ATT_RB - 1) / ATT_RB * (1 + (n_groups > ATT_CB ? (n_groups - ATT_CB + 7) / 8 : 0));
        if (trips1 <= trips2) {
            for (int p0 = hw; p0 < n_pairs; p0 += ATT_GW) attn_merge_rows<T, H, 1, ATT_CB1>(a, head, p0, n_pairs, pos0, lane);
        } else {
            for (int p0 = hw * ATT_RB; p0 < n_pairs; p0 += ATT_GW * ATT_RB) attn_merge_rows<T, H>(a, head, p0, n_pairs, pos0, lane);
        }
    }
    __syncthreads();
}

// Workgroup -> (group, first head) of the per-step kernels.  Workgroups are handed to the 8 XCDs round robin by index, and
// each XCD has its own L2: the query heads that share a KV head (grouped-query attention) read the same K/V, so the
// workgroups of one (KV head, group) pair get consecutive slots of ONE XCD and its K/V crosses the fabric once instead
// of once per query head; successive pairs go to successive XCDs.  Returns false for the padding workgroups of the last round.
__device__ __forceinline__ bool attn_unit(const AttnArgs& a, const int index, int* grp, int* head) {
    const int xcd = index & 7, slot = index >> 3, G = a.n_h / a.n_kv, U = G / a.gh;   // U workgroups per pair
    const int pair = (slot / U) * 8 + xcd;
    if (pair >= a.n_kv * a.grid_groups) return false;
    // pairs in group-major order: the launch sweeps the cache page by page (a page's KV heads are neighbours in
    // memory), and the workgroups dispatched last are the heads' last, partly filled groups, so the short final round
    // of a long context is light (8K context: 36 -> 33 us)
    *grp = pair / a.n_kv;
    *head = (pair % a.n_kv) * G + (slot % U) * a.gh;
    return true;
}
__host__ __device__ inline int attn_grid(int n_h, int n_kv, int groups, int gh) { return (n_kv * groups + 7) / 8 * 8 * (n_h / n_kv / gh); }

// The leading scalar parameters of the two kernels repeat what a wave needs before its first requests: built with
// kernel-argument preloading they arrive in SGPRs with the wave, while the argument structure comes from memory.
// heads = n_h | n_kv << 16, rows = M | RS << 8 | gh << 16.
#define ATT_HOT_PARAMS const void* q, const void* kv, const int32_t* page_table, int64_t q_plane, int32_t heads, int32_t rows, \
                       int32_t grid_groups, int32_t cap_chunks, int32_t page_tokens, int32_t
#define ATT_HOT_ARGS(a0)                                                                                                   \
    AttnArgs a = a0;                                                                                                       \
    a.q = q; a.kv = kv; a.page_table = page_table; a.q_plane = q_plane; a.n_h = heads & 0xffff; a.n_kv = heads >> 16;      \
    a.M = rows & 255; a.RS = (rows >> 8) & 255; a.gh = rows >> 16; a.grid_groups = grid_groups; a.cap_chunks = cap_chunks; \
    a.page_tokens = page_tokens;
template <class T, int H>
__global__ __launch_bounds__(ATT_GW * 64) void attn_kernel(ATT_HOT_PARAMS, const AttnArgs a0) {
    ATT_HOT_ARGS(a0)
    __shared__ float so[ATT_GW * ATT_RH * H];
    __shared__ float sml[ATT_GW * ASD_ROWS * 2];
    __shared__ unsigned s_old;
    int grp, head;
    if (!attn_unit(a, blockIdx.x, &grp, &head)) return;
    // (a group no row of this call sees does nothing: every wave of it is inactive, and a context of one group
    // returns before the arrival)
    attn_group<T, H, true>(a, grp, head, true, __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), threadIdx.x & 63, so, sml, &s_old);
}

// The same kernel with the register allocation held to four waves per SIMD (128 registers instead of ~220): a wave
// then no longer keeps all of a chunk's K and V^T fragments in flight at once, but every group of a long context is
// resident at once (one round of workgroups instead of two).  Same arithmetic, same bits; chosen by the grid size.
template <class T, int H>
__global__ __launch_bounds__(ATT_GW * 64, 4) void attn_kernel_w4(ATT_HOT_PARAMS, const AttnArgs a0) {
    ATT_HOT_ARGS(a0)
    __shared__ float so[ATT_GW * ATT_RH * H];
    __shared__ float sml[ATT_GW * ASD_ROWS * 2];
    __shared__ unsigned s_old;
    int grp, head;
    if (!attn_unit(a, blockIdx.x, &grp, &head)) return;
    if (grp * ATT_GROUP > a.st->pos + a.pos_off + a.M - 1) return;
    attn_group<T, H>(a, grp, head, true, __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), threadIdx.x & 63, so, sml, &s_old);
}

// ---------------------------------------------------------------- prompt blocks: causal attention
// 16 * PF_ATT_NT query rows of a prompt block (cache positions pos0 + ...) of one query head against all keys up to
// their own positions.  Same fragments and key order as the decode kernel above.  Workgroups are numbered longest
// row block first.
struct PfAttnArgs {
    const void* q;            // [chunk][n_h*h/KE][16][KE], planes q_plane elements apart, chunks q_chunk apart
    void* out;                // same layout
    int64_t q_plane, q_chunk;
    const void* kv;
    const int32_t* page_table;
    int32_t pos0, rows;       // cache position of row 0 of the block, valid rows
    int32_t n_h, n_kv, h, page_tokens;
    float scale;
};

#ifndef PF_ATT_NT
#define PF_ATT_NT 2            // 16-row chunks of query rows per workgroup of pf_attn_kernel
#endif
// A workgroup takes 32 query rows (two 16-row chunks) and splits the keys over its four waves: wave w walks the
// 64-key chunks w, w + 4, ... with a running maximum and sum per row (the output accumulator is rescaled when the
// maximum grows), and the four partial results are merged through LDS in wave order at the end, so the result has
// one fixed order.  A chunk's K and V^T fragments are loaded once per 32 query rows and feed two column tiles of
// matrix-core work (with one tile per load the loads, not the products, fill the time: 1.8x slower at 8K context);
// the next chunk's K fragments are requested as soon as the score products have consumed the current ones, the
// next V^T fragments right after the output products, into the same registers (the scheduler is fenced at those
// points: without the fences, or with three column tiles, the kernel is slower).  Needs a SIMD's whole register
// file per wave.
template <class T, int H>
__global__ __launch_bounds__(256, 1) void pf_attn_kernel(const PfAttnArgs a) {
    using E = typename T::elem;
    constexpr int KE = T::KE, HS = H / (4 * KE), HT = H / 16, KST = 64 / (4 * KE), NP = T::NP, NT = PF_ATT_NT, NWV = 4;
    __shared__ float so[NWV][16][H];
    __shared__ float sml[NWV][NT][16][2];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, g = lane >> 4, m = lane & 15, r = lane & 15;
    const int n_units = (a.rows + 16 * NT - 1) / (16 * NT);
    const int u = n_units - 1 - (int)blockIdx.x, head = blockIdx.y;
    const int rows_u = min(16 * NT, a.rows - 16 * NT * u);
    const int p0 = a.pos0 + 16 * NT * u, last = p0 + rows_u - 1;
    const int kvh = head / (a.n_h / a.n_kv), PT = a.page_tokens;
    int M[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) M[t] = min(16, max(0, rows_u - 16 * t));

    u32x4 qf[NT][HS][NP];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const E* qp = (const E*)a.q + (size_t)(NT * u + t) * a.q_chunk + (size_t)head * H * 16;
#pragma unroll
        for (int hs = 0; hs < HS; ++hs)
#pragma unroll
            for (int pl = 0; pl < NP; ++pl)
                qf[t][hs][pl] = m < M[t] ? *(const u32x4*)(qp + pl * a.q_plane + ((size_t)(hs * 4 + g) * 16 + m) * KE) : u32x4{0u, 0u, 0u, 0u};
    }
    f32x4 o[NT][HT];
    float mx[NT], l[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        mx[t] = -INFINITY; l[t] = 0.f;
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) o[t][ht] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    u32x4 kf[4][HS], vf[HT][KST];
    auto chunk_base = [&](int kcv) {        // this lane's pointer into chunk kc of the cache block (K fragments, then V^T fragments)
        // the chunk index is the same in every lane: as a scalar read through the constant address space (nothing
        // writes the page table while a pass runs) the page lookup is a scalar load, outside the vector loads' queue
        typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
        const int kc = __builtin_amdgcn_readfirstlane(kcv);
        const int page = ((const_i32_ptr)(uintptr_t)a.page_table)[(kc * ASD_CHUNK) / PT], slot0 = (kc * ASD_CHUNK) % PT;
        return (const E*)a.kv + ((size_t)page * a.n_kv + kvh) * 2 * PT * H + kv_chunk_off<T>(slot0 / ASD_CHUNK, H) + lane * KE;
    };
    auto issue_k = [&](const E* Kc) {
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int hs = 0; hs < HS; ++hs)
                kf[kt][hs] = *(const u32x4*)(Kc + kv_k_frag_off<T>(kt, hs, H));
    };
    auto issue_v = [&](const E* Kc, int) {
#pragma unroll
        for (int ht = 0; ht < HT; ++ht)
#pragma unroll
            for (int ks = 0; ks < KST; ++ks)
                vf[ht][ks] = *(const u32x4*)(Kc + kv_v_frag_off<T>(ht, ks, H));
    };
    auto one_chunk = [&](const int kc, auto has_next) {
        constexpr bool more = decltype(has_next)::value;
        const E* Kn = nullptr;
        if constexpr (more) Kn = chunk_base(kc + NWV);
        f32x4 s[NT][4];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
                s[t][kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int hs = 0; hs < HS; ++hs)
#pragma unroll
                    for (int pl = 0; pl < NP; ++pl) mma16<T>(s[t][kt], kf[kt][hs], qf[t][hs][pl]);
            }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (more) issue_k(Kn);                 // the K registers are free again
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            // causal mask, running maximum and sum per row (= per column m); a chunk none of whose keys a row sees
            // leaves that row's state as it is
            const int row_pos = p0 + 16 * t + m;
            float cm = -INFINITY;
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int key = kc * ASD_CHUNK + score_key<T>(kt, 4 * g + j);
                    const float v = (key <= row_pos) ? s[t][kt][j] * a.scale : -INFINITY;
                    s[t][kt][j] = v;
                    cm = fmaxf(cm, v);
                }
            cm = fmaxf(cm, __shfl_xor(cm, 16));
            cm = fmaxf(cm, __shfl_xor(cm, 32));
            const float mn = fmaxf(mx[t], cm);
            const float alpha = (mx[t] == -INFINITY) ? 0.f : __expf(mx[t] - mn);
            float cs = 0.f;
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float p = (s[t][kt][j] == -INFINITY) ? 0.f : __expf(s[t][kt][j] - mn);
                    s[t][kt][j] = p;
                    cs += p;
                }
            cs += __shfl_xor(cs, 16);
            cs += __shfl_xor(cs, 32);
            l[t] = l[t] * alpha + cs;
            mx[t] = mn;
#pragma unroll
            for (int ht = 0; ht < HT; ++ht) { o[t][ht][0] *= alpha; o[t][ht][1] *= alpha; o[t][ht][2] *= alpha; o[t][ht][3] *= alpha; }
            u32x4 pf[KST][NP];
            att_pfrags<T>(s[t], pf);
#pragma unroll
            for (int ht = 0; ht < HT; ++ht)
#pragma unroll
                for (int ks = 0; ks < KST; ++ks)
#pragma unroll
                    for (int pl = 0; pl < NP; ++pl) mma16<T>(o[t][ht], vf[ht][ks], pf[ks][pl]);
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (more) issue_v(Kn, kc + NWV);       // and so are the V^T registers
        __builtin_amdgcn_sched_barrier(0);
    };

    const int n_kc = last / ASD_CHUNK + 1;
    if (w < n_kc) {
        const E* Kc = chunk_base(w);
        issue_k(Kc);
        issue_v(Kc, w);
        int kc = w;
        for (; kc + NWV < n_kc; kc += NWV) one_chunk(kc, std::true_type{});
        one_chunk(kc, std::false_type{});
    }

    // ---- merge the four waves' partial results, wave order, one 16-row chunk at a time
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        if (g == 0) { sml[w][t][m][0] = mx[t]; sml[w][t][m][1] = l[t]; }
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) *(f32x4*)&so[w][m][ht * 16 + 4 * g] = o[t][ht];
        __syncthreads();
        const int row = tid & 15;
        float gmax = -INFINITY;                          // finite: wave 0 holds chunk 0, whose key 0 every row sees
#pragma unroll
        for (int ww = 0; ww < NWV; ++ww) gmax = fmaxf(gmax, sml[ww][t][row][0]);
        float wgt[NWV], L = 0.f;
#pragma unroll
        for (int ww = 0; ww < NWV; ++ww) { wgt[ww] = __expf(sml[ww][t][row][0] - gmax); L += sml[ww][t][row][1] * wgt[ww]; }
        const float inv = 1.f / L;
        for (int d = (tid >> 4) * 4; d < H; d += 64) {
            float v[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ww = 0; ww < NWV; ++ww) {
                const f32x4 x = *(const f32x4*)&so[ww][row][d];
                v[0] += x[0] * wgt[ww]; v[1] += x[1] * wgt[ww]; v[2] += x[2] * wgt[ww]; v[3] += x[3] * wgt[ww];
            }
            v[0] *= inv; v[1] *= inv; v[2] *= inv; v[3] *= inv;
            if (row < M[t]) store_act4<T>(a.out, a.q_plane, (int64_t)(NT * u + t) * a.q_chunk, head * H + d, row, v);
        }
        __syncthreads();
    }
}
