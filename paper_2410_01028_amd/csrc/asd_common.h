// Common device-side definitions: storage types, the 16-byte MFMA fragment, layouts.
//
// Layouts (KE = elements per 16-byte fragment: 8 for bf16, 4 for fp32; one
// "k-block" = 4*KE consecutive k values = what one fragment step of a wave covers):
//
//  * tiled weight  W[N][K] -> [N/16 tiles][KB k-blocks][64 lanes][KE]
//      lane = 16*g + r holds row 16*tile + r, k = kb*4*KE + g*KE .. +KE   (K padded with 0 to KB*4*KE)
//    so that one wave reads one contiguous KiB per step and a tile's K range is
//    one contiguous stream in HBM;
//  * tiled activation X[rows][K] -> [K/KE][RS][KE] with RS = the pass's row stride (its row count): the
//    fragment of k-block kb for lane 16*g + m is the 16 bytes at ((kb*4 + g)*RS + m)*KE; lanes of unused
//    rows read row 0 (their columns of the products are never looked at), so a one-row pass reads 64 bytes
//    of activations per KiB of weights;
//  * KV cache: per (page, KV head) and 64-key chunk the K fragments, then the V^T fragments, each the
//    contiguous 1 KiB register image of one attention load (see kv_k_off / kv_v_off below).
//
// MFMA operand use: A = weights (16 output features x k-block), B = activations
// (k-block x 16 rows), D[n][m]: lane 16*g + m holds n = 4*g + j in register j.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

// planes of a bf16 activation (2 = hi + lo; 1 is a build-time experiment: single bf16 activations)
#ifndef ASD_BF16_PLANES
#define ASD_BF16_PLANES 2
#endif
#define ASD_WAVE 64
#define ASD_ROWS 16          // rows (MFMA columns) of every forward call
#define ASD_CHUNK 64         // keys per attention work item; chunk boundaries are absolute positions

// NP = planes of an activation buffer: bf16 activations are kept as hi + lo (x ~ hi + lo, lo = bf16(x - hi)) and
// contracted plane by plane, so that what the matrix cores see of an activation carries ~16 mantissa bits;
// weights and the KV cache stay single bf16 values.
struct BF16 {
    using elem = uint16_t;
    static constexpr int KE = 8;
    static constexpr int NP = ASD_BF16_PLANES;
    static __device__ __forceinline__ float to_f32(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
    static __device__ __forceinline__ uint16_t from_f32(float f) {
        return __builtin_bit_cast(uint16_t, (__bf16)f);     // round to nearest even
    }
};
struct F32 {
    using elem = float;
    static constexpr int KE = 4;
    static constexpr int NP = 1;
    static __device__ __forceinline__ float to_f32(float v) { return v; }
    static __device__ __forceinline__ float from_f32(float f) { return f; }
};

// ---- KV cache block of one (page, KV head): page_tokens / 64 chunks of 64 keys; a chunk holds its K fragments, then
// its V^T fragments, and a fragment is the 1 KiB register image of one load instruction (lane 16g + r holds KE
// consecutive elements), so that every attention load reads one contiguous KiB (whole cache lines: a compute unit's
// load path is bound by the number of lines an instruction touches, and 64-byte row segments cost twice as many):
//   K fragment (kt, hs):   lane (g, r) = key score_key(kt, r) of the chunk, head dims hs * 4KE + g * KE ...
//   V^T fragment (ht, ks): lane (g, r) = head dim ht * 16 + r, keys ks * 4KE + g * KE ... of the chunk
// key (0..63, relative to the chunk) held by score tile kt, tile row r: chosen per storage type so that the score
// registers of a lane are exactly the keys of one V^T fragment's lane
template <class T> __device__ __forceinline__ int score_key(int kt, int r);
template <> __device__ __forceinline__ int score_key<BF16>(int kt, int r) {
    return 32 * (kt >> 1) + 8 * (r >> 2) + 4 * (kt & 1) + (r & 3);    // two tiles interleave into one 32-key block
}
template <> __device__ __forceinline__ int score_key<F32>(int kt, int r) { return 16 * kt + r; }
// the inverse: score tile and tile row of a chunk's key
template <class T> __host__ __device__ __forceinline__ void score_tile_of(int key, int* kt, int* r);
template <> __host__ __device__ __forceinline__ void score_tile_of<BF16>(int key, int* kt, int* r) {
    *kt = 2 * (key >> 5) + ((key >> 2) & 1); *r = 4 * ((key >> 3) & 3) + (key & 3);
}
template <> __host__ __device__ __forceinline__ void score_tile_of<F32>(int key, int* kt, int* r) { *kt = key >> 4; *r = key & 15; }
// element offsets inside a block (h = head dim, slot = token slot in the page)
template <class T> __host__ __device__ __forceinline__ size_t kv_chunk_off(int chunk_in_page, int h) { return (size_t)chunk_in_page * 2 * ASD_CHUNK * h; }
template <class T> __host__ __device__ __forceinline__ size_t kv_k_frag_off(int kt, int hs, int h) {      // + lane * KE
    return (size_t)(kt * (h / (4 * T::KE)) + hs) * 64 * T::KE;
}
template <class T> __host__ __device__ __forceinline__ size_t kv_v_frag_off(int ht, int ks, int h) {      // + lane * KE
    return (size_t)ASD_CHUNK * h + (size_t)(ht * (ASD_CHUNK / (4 * T::KE)) + ks) * 64 * T::KE;
}
template <class T> __host__ __device__ __forceinline__ size_t kv_k_off(int slot, int dim, int h) {
    constexpr int KE = T::KE;
    int kt, r;
    score_tile_of<T>(slot % ASD_CHUNK, &kt, &r);
    return kv_chunk_off<T>(slot / ASD_CHUNK, h) + kv_k_frag_off<T>(kt, dim / (4 * KE), h) + (size_t)(((dim / KE) & 3) * 16 + r) * KE + dim % KE;
}
template <class T> __host__ __device__ __forceinline__ size_t kv_v_off(int slot, int dim, int h) {
    constexpr int KE = T::KE;
    const int key = slot % ASD_CHUNK;
    return kv_chunk_off<T>(slot / ASD_CHUNK, h) + kv_v_frag_off<T>(dim >> 4, key / (4 * KE), h) + (size_t)(((key / KE) & 3) * 16 + (dim & 15)) * KE + key % KE;
}

// acc[n][m] += sum over the k-block of A[n][k] * B[k][m]; both fragments use the same lane -> k map.
template <class T> __device__ __forceinline__ void mma16(f32x4& acc, const u32x4& a, const u32x4& b);
template <> __device__ __forceinline__ void mma16<BF16>(f32x4& acc, const u32x4& a, const u32x4& b) {
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}
template <> __device__ __forceinline__ void mma16<F32>(f32x4& acc, const u32x4& a, const u32x4& b) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a[j]), __uint_as_float(b[j]), acc, 0, 0, 0);
}

// element offset of (row m, feature k) in a tiled activation buffer with row stride rs
template <class T> __device__ __forceinline__ size_t act_index(int k, int m, int rs) {
    return ((size_t)(k / T::KE) * rs + m) * T::KE + (k % T::KE);
}

// write value v of (feature k, row m) into every plane of a tiled activation buffer (plane stride in elements)
template <class T>
__device__ __forceinline__ void store_act(void* base, size_t plane, int rs, int k, int m, float v) {
    typename T::elem* p = (typename T::elem*)base + act_index<T>(k, m, rs);
    const typename T::elem hi = T::from_f32(v);
    *p = hi;
    if constexpr (T::NP == 2) p[plane] = T::from_f32(v - T::to_f32(hi));
}

// four consecutive features n0..n0+3 (n0 % 4 == 0) of row m of one chunk, all planes
template <class T>
__device__ __forceinline__ void store_act4(void* base, int64_t plane, int64_t chunk_off, int n0, int m, const float (&v)[4]) {
    using E = typename T::elem;
    E* p = (E*)base + chunk_off + act_index<T>(n0, m, 16);
    if constexpr (sizeof(E) == 2) {
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            hi[j] = T::from_f32(v[j]);
            lo[j] = T::from_f32(v[j] - T::to_f32((uint16_t)hi[j]));
        }
        *(uint2*)p = uint2{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16)};
        if constexpr (T::NP == 2) *(uint2*)(p + plane) = uint2{lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)};
    } else {
        *(float4*)p = float4{v[0], v[1], v[2], v[3]};
    }
}
// Device-resident decoding state, read by kernels so that captured graphs can be replayed unchanged.
struct DevState {
    int32_t pos;        // committed cache length = position of the first row of a verify pass
    int32_t emitted;    // tokens written to the output buffer so far
    int32_t target;     // tokens to emit in this decode call
    int32_t cycles, drafted, accepted;
    float conf;         // top-1 probability of the token the last draft step produced (softmax of its logits)
    int32_t index_base; // sampled decoding: output index of the first token this decode call emits
    int32_t err;        // DEV_ERR_* bits raised by kernels since the state was last set (checked by the host at its next read)
};
// a token id outside the vocabulary reached the embedding (it was replaced by token 0); a row's logits held no
// finite maximum (NaN / Inf weights: the row's greedy token was replaced by token 0)
enum { DEV_ERR_TOKEN = 1, DEV_ERR_LOGITS = 2 };
