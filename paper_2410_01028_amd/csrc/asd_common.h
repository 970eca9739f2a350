// Common device-side definitions: storage types, the 16-byte MFMA fragment, layouts.
//
// Layouts (KE = elements per 16-byte fragment: 8 for bf16, 4 for fp32; one
// "k-block" = 4*KE consecutive k values = what one fragment step of a wave covers):
//
//  * tiled weight  W[N][K] -> [N/16 tiles][KB k-blocks][64 lanes][KE]
//      lane = 16*g + r holds row 16*tile + r, k = kb*4*KE + g*KE .. +KE   (K padded with 0 to KB*4*KE)
//    so that one wave reads one contiguous KiB per step and a tile's K range is
//    one contiguous stream in HBM;
//  * tiled activation X[16 rows][K] -> [K/KE][16 rows][KE]: the fragment of k-block kb
//    for lane 16*g + m is the 16 bytes at ((kb*4 + g)*16 + m)*KE, again one KiB per step.
//
// MFMA operand use: A = weights (16 output features x k-block), B = activations
// (k-block x 16 rows), D[n][m]: lane 16*g + m holds n = 4*g + j in register j.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

#define ASD_WAVE 64
#define ASD_ROWS 16          // rows (MFMA columns) of every forward call
#define ASD_CHUNK 64         // keys per attention work item; chunk boundaries are absolute positions

struct BF16 {
    using elem = uint16_t;
    static constexpr int KE = 8;
    static __device__ __forceinline__ float to_f32(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
    static __device__ __forceinline__ uint16_t from_f32(float f) {
        return __builtin_bit_cast(uint16_t, (__bf16)f);     // round to nearest even
    }
};
struct F32 {
    using elem = float;
    static constexpr int KE = 4;
    static __device__ __forceinline__ float to_f32(float v) { return v; }
    static __device__ __forceinline__ float from_f32(float f) { return f; }
};

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

// element offset of (row m, feature k) in a tiled activation buffer
template <class T> __device__ __forceinline__ size_t act_index(int k, int m) {
    return ((size_t)(k / T::KE) * ASD_ROWS + m) * T::KE + (k % T::KE);
}

// Device-resident decoding state, read by kernels so that captured graphs can be replayed unchanged.
struct DevState {
    int32_t pos;        // committed cache length = position of the first row of a verify pass
    int32_t emitted;    // tokens written to the output buffer so far
    int32_t target;     // tokens to emit in this decode call
    int32_t cycles, drafted, accepted;
    int32_t pad[2];
};
