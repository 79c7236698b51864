// Pieces shared by the two W4A16 GEMM kernels (matrix-core prefill kernel, skinny decode kernel):
// kernel arguments, the packed-fp16 int4 dequantizer and the fragment -> weight-matrix mapping.
#pragma once
#include "qtale_dev.h"
#include "qtale_kernels.h"

namespace qtale {

struct GemmDev {
    const half_t* A;
    const int32_t* count;
    int M_max, K, KT, gshift;
    const U4* codes[3];
    const uint32_t* sz[3];
    int N[3], NF[3], npad[3], colbase[3];
    int n_w, vf_total, tiles_m, tiles_n;
    void* out;
    int ldo;
    const void* resid;
    const int32_t* idx;
    int bf16;
};

constexpr int kLdsStride = 72;     // halves per LDS row of the A tile (64 + 8 padding)

// (x & mask) | magic in ONE VALU op.  gfx9 VOP3 encodings take no literal and at most one scalar operand,
// so the compiler falls back to v_and_b32 + v_or_b32 with two literals; with the mask in an SGPR and the
// magic constant pinned in a VGPR, v_and_or_b32 is legal.
__device__ __forceinline__ uint32_t and_or(uint32_t x, uint32_t mask_sgpr, uint32_t magic_vgpr) {
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "s"(mask_sgpr), "v"(magic_vgpr));
    return r;
}

// 8 packed int4 codes of one prepacked word -> 8 fp16 weights (c - z) * s, bit-identical to fp16((c-z)*s):
// OR-ing a nibble into 0x6400 gives 1024 + c (nibble at bits 0-3 of a half) or 1024 + 16 c (bits 4-7).
__device__ __forceinline__ half8_t dequant8(uint32_t w, half2_t S, half2_t Zlo, half2_t Zhi, uint32_t magic) {
    const half2_t sixteenth = {static_cast<half_t>(0.0625f), static_cast<half_t>(0.0625f)};
    const uint32_t w8 = w >> 8;
    const half2_t l0 = __builtin_bit_cast(half2_t, and_or(w, 0x000f000fu, magic));
    const half2_t h0 = __builtin_bit_cast(half2_t, and_or(w, 0x00f000f0u, magic));
    const half2_t l1 = __builtin_bit_cast(half2_t, and_or(w8, 0x000f000fu, magic));
    const half2_t h1 = __builtin_bit_cast(half2_t, and_or(w8, 0x00f000f0u, magic));
    const half2_t p0 = (l0 - Zlo) * S;
    const half2_t p1 = __builtin_elementwise_fma(h0, sixteenth, -Zhi) * S;
    const half2_t p2 = (l1 - Zlo) * S;
    const half2_t p3 = __builtin_elementwise_fma(h1, sixteenth, -Zhi) * S;
    half8_t r;
    r[0] = p0[0]; r[1] = p0[1]; r[2] = p1[0]; r[3] = p1[1];
    r[4] = p2[0]; r[5] = p2[1]; r[6] = p3[0]; r[7] = p3[1];
    return r;
}

// The 0x64006400 constant held in a VGPR (see and_or).
__device__ __forceinline__ uint32_t dequant_magic() {
    uint32_t m;
    asm volatile("v_mov_b32 %0, 0x64006400" : "=v"(m));
    return m;
}

struct ScaleZero {
    half2_t S, Zlo, Zhi;
};
__device__ __forceinline__ ScaleZero expand_sz(uint32_t raw) {
    const half2_t sz = __builtin_bit_cast(half2_t, raw);       // [0] = scale, [1] = zero-point
    ScaleZero r;
    r.S = half2_t{sz[0], sz[0]};
    const half_t zlo = sz[1] + static_cast<half_t>(1024.0f);
    const half_t zhi = sz[1] + static_cast<half_t>(64.0f);
    r.Zlo = half2_t{zlo, zlo};
    r.Zhi = half2_t{zhi, zhi};
    return r;
}

__device__ __forceinline__ float silu_f(float g) { return g / (1.0f + __expf(-g)); }


// Virtual fragment index -> (weight matrix, 32-row fragment inside it).  Gate/up pairs are interleaved
// (even = gate, odd = up) so one wave owns both halves of a SwiGLU output; q|k|v are concatenated.
template <int EPI>
__device__ __forceinline__ void map_fragment(const GemmDev& p, int vf, int& mat, int& f) {
    if (EPI == EPI_SWIGLU_F16) {
        mat = vf & 1;
        f = vf >> 1;
    } else {
        mat = 0;
        f = vf;
        if (p.n_w > 1 && f >= p.NF[0]) { f -= p.NF[0]; mat = 1; }
        if (p.n_w > 2 && mat == 1 && f >= p.NF[1]) { f -= p.NF[1]; mat = 2; }
    }
}

hipError_t launch_gemm_skinny(GemmDev& d, int epilogue, hipStream_t stream);

}  // namespace qtale
