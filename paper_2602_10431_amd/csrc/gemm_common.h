// Pieces shared by the two W4A16 GEMM kernels (matrix-core prefill kernel, skinny decode kernel):
// kernel arguments, the packed-fp16 int4 dequantizer and the fragment -> weight-matrix mapping.
#pragma once
#include "qtale_dev.h"
#include "qtale_kernels.h"

namespace qtale {

struct GemmDev {
    const half_t* A;
    const int32_t* count;
    int M_max, rows_exact, K, KT, gshift;
    const void* codes[3];
    const uint32_t* sz[3];
    int N[3], NF[3], npad[3], colbase[3];
    int n_w, vf_total, tiles_m, tiles_n;
    int row_chunks;                // skinny kernel: 64-row chunks of the activation matrix (1 for M <= 64)
    void* out;
    int ldo;
    const void* resid;
    const int32_t* idx;
    int bf16;
    int bits;                      // 4, 3 or 2: width of the weight codes
    int ksplit;                    // decode kernel: parts K is cut into across workgroups (1 = none)
    int epi_rt;                    // decode kernel: epilogue chosen at run time (GemmEpilogue)
    int tail;                      // 0: all rows; 1: all but gemm_tail_rows(); 2: only those last rows (small-row kernels)
    int M_full;                    // tail == 2: host bound on the row count of the whole matrix (M_max bounds the tail)
    int tail_tiles_n, tail_slots;  // tail != 0: column tiles of the 128-row-tile launch, workgroups the chip holds
};

// Rows the 128-row-tile kernel hands to the small-row kernels: the rows after the last full tile, when leaving their
// row of tiles out saves the launch a whole round of workgroups (tile count / workgroups the chip holds, rounded up).
// Measured on the 7B-shaped layer at 4115 instead of 4096 rows (33 x 16 tiles on 512 slots): down-proj 0.47 -> 0.37
// ms, o-proj 0.20 -> 0.17 ms with the 19 rows as a separate small-row launch; where no round is saved the same split
// costs 10-30 us per linear, so it is not made.  Both launches evaluate this on the device-side count with the
// same tiles_n and slots.
__host__ __device__ inline int gemm_tail_rows(int M, int tiles_n, int slots) {
    const int rem = M & 127, full = M >> 7;
    if (full == 0 || rem == 0) return 0;
    return ((full + 1) * tiles_n + slots - 1) / slots > (full * tiles_n + slots - 1) / slots ? rem : 0;
}

// Small-row kernels: first row and row count of this workgroup's chunk.  chunk_row0 is the start of its chunk inside
// the rows the launch covers: the whole matrix, or (tail launch) the rows after the last full 128-row tile.
__device__ __forceinline__ bool gemm_chunk_rows(const GemmDev& p, int chunk_row0, int rows_per_chunk, int& row0, int& M) {
    if (p.tail == 2) {
        const int full = p.count ? min(*p.count, p.M_full) : p.M_full;
        const int t = gemm_tail_rows(full, p.tail_tiles_n, p.tail_slots);
        row0 = full - t + chunk_row0;
        M = min(t - chunk_row0, rows_per_chunk);
    } else {
        row0 = chunk_row0;
        M = min((p.count ? min(*p.count, p.M_max) : p.M_max) - row0, rows_per_chunk);
    }
    return M > 0;
}

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

// ---- 3-bit codes ------------------------------------------------------------------------------------
// A lane's 32 codes of one fragment x k-tile occupy three words.  Each 16-bit half of a word holds five
// codes at bits 0-2, 3-5, 6-8, 9-11, 12-14; pair h (codes 2h, 2h+1 of the lane, h = 0..14) sits at field
// h%5 of word h/5, the even code in the low half and the odd one in the high half.  Pair 15 is spread over
// the spare bits 15 / 31 of the three words (bit i of the code in word i).  OR-ing a field into 0x6400
// gives 1024 + c, 1024 + 8c or 1024 + 64c; subtracting 1024 + z, or one FMA with 1/8 (1/64) and
// -(128 + z) (-(16 + z)), yields c - z exactly, and the multiply by the scale rounds once.
struct ScaleZero3 {
    half2_t S, Z0, Z3, Z6;
};
__device__ __forceinline__ ScaleZero3 expand_sz3(uint32_t raw) {
    const half2_t sz = __builtin_bit_cast(half2_t, raw);
    ScaleZero3 r;
    r.S = half2_t{sz[0], sz[0]};
    const half_t z0 = sz[1] + static_cast<half_t>(1024.0f);
    const half_t z3 = sz[1] + static_cast<half_t>(128.0f);
    const half_t z6 = sz[1] + static_cast<half_t>(16.0f);
    r.Z0 = half2_t{z0, z0};
    r.Z3 = half2_t{z3, z3};
    r.Z6 = half2_t{z6, z6};
    return r;
}

// Pair h of the lane's tile (h must fold to a constant after unrolling).
__device__ __forceinline__ half2_t dequant_pair3(const u32x3_t& t, int h, const ScaleZero3& s, uint32_t magic) {
    const half2_t eighth = {static_cast<half_t>(0.125f), static_cast<half_t>(0.125f)};
    const half2_t sixtyfourth = {static_cast<half_t>(0.015625f), static_cast<half_t>(0.015625f)};
    if (h == 15) {
        const uint32_t bits = ((t.x >> 15) & 0x00010001u) | ((t.y >> 14) & 0x00020002u) | ((t.z >> 13) & 0x00040004u);
        const half2_t l = __builtin_bit_cast(half2_t, bits | magic);
        return (l - s.Z0) * s.S;
    }
    const int wi = h / 5, f = h % 5;
    const uint32_t w = wi == 0 ? t.x : wi == 1 ? t.y : t.z;
    if (f == 0) return (__builtin_bit_cast(half2_t, and_or(w, 0x00070007u, magic)) - s.Z0) * s.S;
    if (f == 1) return __builtin_elementwise_fma(__builtin_bit_cast(half2_t, and_or(w, 0x00380038u, magic)), eighth, -s.Z3) * s.S;
    if (f == 2) return __builtin_elementwise_fma(__builtin_bit_cast(half2_t, and_or(w, 0x01c001c0u, magic)), sixtyfourth, -s.Z6) * s.S;
    const uint32_t w9 = w >> 9;
    if (f == 3) return (__builtin_bit_cast(half2_t, and_or(w9, 0x00070007u, magic)) - s.Z0) * s.S;
    return __builtin_elementwise_fma(__builtin_bit_cast(half2_t, and_or(w9, 0x00380038u, magic)), eighth, -s.Z3) * s.S;
}

// ---- 2-bit codes -------------------------------------------------------------------------------------
// A lane's 32 codes of one fragment x k-tile occupy two words; pair h (codes 2h, 2h+1) sits in word h/8 at bit
// 2*(h%8) of the low half (even code) and of the high half (odd code).  Fields at bits 0, 2, 4 are OR-ed into
// 0x6400 directly (1024 + c, 1024 + 4c, 1024 + 16c), the others after a shift by 6 or 12.
struct ScaleZero2 {
    half2_t S, Z0, Z1, Z2;
};
__device__ __forceinline__ ScaleZero2 expand_sz2(uint32_t raw) {
    const half2_t sz = __builtin_bit_cast(half2_t, raw);
    ScaleZero2 r;
    r.S = half2_t{sz[0], sz[0]};
    const half_t z0 = sz[1] + static_cast<half_t>(1024.0f);
    const half_t z1 = sz[1] + static_cast<half_t>(256.0f);
    const half_t z2 = sz[1] + static_cast<half_t>(64.0f);
    r.Z0 = half2_t{z0, z0};
    r.Z1 = half2_t{z1, z1};
    r.Z2 = half2_t{z2, z2};
    return r;
}

// Pair h of the lane's tile (h must fold to a constant after unrolling).
__device__ __forceinline__ half2_t dequant_pair2(const u32x2_t& t, int h, const ScaleZero2& s, uint32_t magic) {
    const half2_t quarter = {static_cast<half_t>(0.25f), static_cast<half_t>(0.25f)};
    const half2_t sixteenth = {static_cast<half_t>(0.0625f), static_cast<half_t>(0.0625f)};
    const int slot = h & 7;
    const uint32_t w = (h >> 3) == 0 ? t.x : t.y;
    const uint32_t src = slot < 3 ? w : slot < 6 ? (w >> 6) : (w >> 12);
    const int f = slot < 3 ? slot : slot < 6 ? slot - 3 : slot - 6;
    if (f == 0) return (__builtin_bit_cast(half2_t, and_or(src, 0x00030003u, magic)) - s.Z0) * s.S;
    if (f == 1) return __builtin_elementwise_fma(__builtin_bit_cast(half2_t, and_or(src, 0x000c000cu, magic)), quarter, -s.Z1) * s.S;
    return __builtin_elementwise_fma(__builtin_bit_cast(half2_t, and_or(src, 0x00300030u, magic)), sixteenth, -s.Z2) * s.S;
}

// ---- the code widths behind one interface ---------------------------------------------------------------
// WBits<BITS>: register type of a lane's packed codes for one fragment x k-tile, bytes per lane, expanded
// scale/zero constants, the load and the dequantisation of k-step j (8 weights in operand order).
template <int BITS>
struct WBits;

template <>
struct WBits<4> {
    using Tile = u32x4_t;
    using SZ = ScaleZero;
    static constexpr int kLaneBytes = 16;
    static __device__ __forceinline__ Tile load(const void* frag_base, int kt, int lane) {
        return (reinterpret_cast<const u32x4_t*>(frag_base) + static_cast<size_t>(kt) * 64)[lane];
    }
    static __device__ __forceinline__ Tile load_lane(const char* lane_ptr) { return *reinterpret_cast<const u32x4_t*>(lane_ptr); }
    static __device__ __forceinline__ SZ expand(uint32_t raw) { return expand_sz(raw); }
    static __device__ __forceinline__ half8_t dequant(const Tile& t, int j, const SZ& s, uint32_t magic) {
        const uint32_t w = j == 0 ? t.x : j == 1 ? t.y : j == 2 ? t.z : t.w;
        return dequant8(w, s.S, s.Zlo, s.Zhi, magic);
    }
};

template <>
struct WBits<2> {
    using Tile = u32x2_t;
    using SZ = ScaleZero2;
    static constexpr int kLaneBytes = 8;
    static __device__ __forceinline__ Tile load(const void* frag_base, int kt, int lane) {
        return (reinterpret_cast<const u32x2_t*>(frag_base) + static_cast<size_t>(kt) * 64)[lane];
    }
    static __device__ __forceinline__ Tile load_lane(const char* lane_ptr) { return *reinterpret_cast<const u32x2_t*>(lane_ptr); }
    static __device__ __forceinline__ SZ expand(uint32_t raw) { return expand_sz2(raw); }
    static __device__ __forceinline__ half8_t dequant(const Tile& t, int j, const SZ& s, uint32_t magic) {
        const half2_t p0 = dequant_pair2(t, 4 * j + 0, s, magic);
        const half2_t p1 = dequant_pair2(t, 4 * j + 1, s, magic);
        const half2_t p2 = dequant_pair2(t, 4 * j + 2, s, magic);
        const half2_t p3 = dequant_pair2(t, 4 * j + 3, s, magic);
        half8_t r;
        r[0] = p0[0]; r[1] = p0[1]; r[2] = p1[0]; r[3] = p1[1];
        r[4] = p2[0]; r[5] = p2[1]; r[6] = p3[0]; r[7] = p3[1];
        return r;
    }
};

template <>
struct WBits<3> {
    using Tile = u32x3_t;
    using SZ = ScaleZero3;
    static constexpr int kLaneBytes = 12;
    static __device__ __forceinline__ Tile load(const void* frag_base, int kt, int lane) {
        const uint32_t* p = reinterpret_cast<const uint32_t*>(frag_base) + (static_cast<size_t>(kt) * 64 + lane) * 3;
        Tile t;
        t.x = p[0]; t.y = p[1]; t.z = p[2];
        return t;
    }
    static __device__ __forceinline__ Tile load_lane(const char* lane_ptr) {
        const uint32_t* p = reinterpret_cast<const uint32_t*>(lane_ptr);
        Tile t;
        t.x = p[0]; t.y = p[1]; t.z = p[2];
        return t;
    }
    static __device__ __forceinline__ SZ expand(uint32_t raw) { return expand_sz3(raw); }
    static __device__ __forceinline__ half8_t dequant(const Tile& t, int j, const SZ& s, uint32_t magic) {
        const half2_t p0 = dequant_pair3(t, 4 * j + 0, s, magic);
        const half2_t p1 = dequant_pair3(t, 4 * j + 1, s, magic);
        const half2_t p2 = dequant_pair3(t, 4 * j + 2, s, magic);
        const half2_t p3 = dequant_pair3(t, 4 * j + 3, s, magic);
        half8_t r;
        r[0] = p0[0]; r[1] = p0[1]; r[2] = p1[0]; r[3] = p1[1];
        r[4] = p2[0]; r[5] = p2[1]; r[6] = p3[0]; r[7] = p3[1];
        return r;
    }
};

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

// Epilogue of the tiled kernels.  A wave holds FM x FN accumulator fragments (rows row_base + fm*32 ...,
// virtual fragments vf0 ... vf0 + FN - 1).  Accumulator register r of a lane holds C[row][col] with
// col = lane%32 and row = 8*(r/4) + 4*(lane/32) + r%4 inside a 32x32 fragment.  The wave transposes one
// 32-row slab at a time through its private LDS region `Cs` (32 x (columns + 8) floats) so that global
// traffic is row-contiguous: a lane then owns 4 consecutive columns of one row (16-byte fp32 / 8-byte
// 16-bit accesses, 128+ contiguous bytes per row per wave).  The four epilogues fuse what follows the
// linear: fp16 store (q|k|v), residual add from the gathered rows of x into an fp32 h (o-proj),
// SiLU(gate)*up (MLP), residual add + scatter back into x (down-proj).
template <int EPI, int FM, int FN>
__device__ __forceinline__ void store_tile(const GemmDev& p, const float16_t (&acc)[FM][FN], float* Cs, int lane,
                                           int row_base, int vf0, int M) {
    constexpr int NFO = EPI == EPI_SWIGLU_F16 ? FN / 2 : FN;   // output fragments per wave
    constexpr int CW = NFO * 32;                               // output columns per wave
    constexpr int CSTR = CW + 8;                               // slab row stride (floats): conflict-free writes
    constexpr int LPR = CW / 4;                                // lanes per row when reading back
    constexpr int RPP = 64 / LPR;                              // rows per pass
    constexpr int PASSES = 32 / RPP;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int rr = lane / LPR;                                 // row inside a pass
    const int c4 = (lane % LPR) * 4;                           // first of this lane's 4 columns in the slab
    // which output fragment / matrix the lane's columns belong to
    const int fo = c4 >> 5;
    const int o_vf = vf0 + (EPI == EPI_SWIGLU_F16 ? 2 * fo : fo);
    const bool o_valid = o_vf < p.vf_total;
    int o_mat = 0, o_f = o_vf;
    map_fragment<EPI>(p, o_vf, o_mat, o_f);
    const int o_ncol = o_f * 32 + (c4 & 31);
    const bool col_ok = o_valid && o_ncol < p.N[o_mat];        // N % 4 == 0: the 4 columns are all in or all out
    const int col = (EPI == EPI_SWIGLU_F16 ? 0 : p.colbase[o_mat]) + o_ncol;
    const int32_t* __restrict__ idx = p.idx;

#pragma unroll
    for (int fm = 0; fm < FM; ++fm) {
#pragma unroll
        for (int f = 0; f < NFO; ++f) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float v;
                if (EPI == EPI_SWIGLU_F16) v = silu_f(acc[fm][2 * f][r]) * acc[fm][2 * f + 1][r];
                else v = acc[fm][f][r];
                Cs[(8 * (r >> 2) + 4 * lhi + (r & 3)) * CSTR + f * 32 + l32] = v;
            }
        }
        const int row0 = row_base + fm * 32 + rr;
#pragma unroll
        for (int ps = 0; ps < PASSES; ps += 4) {
            float4 v[4], res[4];
            uint2 xr[4];
            int trow[4];
            bool ok[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int row = row0 + (ps + u) * RPP;
                ok[u] = col_ok && row < M;
                v[u] = *reinterpret_cast<const float4*>(&Cs[((ps + u) * RPP + rr) * CSTR + c4]);
                trow[u] = row;
                if (EPI == EPI_RESID_F32 || EPI == EPI_RESID_SCATTER) trow[u] = ok[u] ? idx[row] : 0;
            }
            if (EPI == EPI_RESID_F32) {
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (ok[u]) xr[u] = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(p.resid) + static_cast<size_t>(trow[u]) * p.ldo + col);
            } else if (EPI == EPI_RESID_SCATTER) {
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (ok[u]) res[u] = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(p.resid) + static_cast<size_t>(row0 + (ps + u) * RPP) * p.ldo + col);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (!ok[u]) continue;
                const int row = row0 + (ps + u) * RPP;
                if (EPI == EPI_STORE_F16 || EPI == EPI_SWIGLU_F16) {
                    uint2 o;
                    o.x = static_cast<uint32_t>(float_to_half_bits(v[u].x)) | (static_cast<uint32_t>(float_to_half_bits(v[u].y)) << 16);
                    o.y = static_cast<uint32_t>(float_to_half_bits(v[u].z)) | (static_cast<uint32_t>(float_to_half_bits(v[u].w)) << 16);
                    *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(p.out) + static_cast<size_t>(row) * p.ldo + col) = o;
                } else if (EPI == EPI_RESID_F32) {
                    float4 o;
                    o.x = act_to_float(static_cast<uint16_t>(xr[u].x & 0xffffu), p.bf16) + v[u].x;
                    o.y = act_to_float(static_cast<uint16_t>(xr[u].x >> 16), p.bf16) + v[u].y;
                    o.z = act_to_float(static_cast<uint16_t>(xr[u].y & 0xffffu), p.bf16) + v[u].z;
                    o.w = act_to_float(static_cast<uint16_t>(xr[u].y >> 16), p.bf16) + v[u].w;
                    *reinterpret_cast<float4*>(reinterpret_cast<float*>(p.out) + static_cast<size_t>(row) * p.ldo + col) = o;
                } else {
                    uint2 o;
                    o.x = static_cast<uint32_t>(float_to_act(res[u].x + v[u].x, p.bf16)) |
                          (static_cast<uint32_t>(float_to_act(res[u].y + v[u].y, p.bf16)) << 16);
                    o.y = static_cast<uint32_t>(float_to_act(res[u].z + v[u].z, p.bf16)) |
                          (static_cast<uint32_t>(float_to_act(res[u].w + v[u].w, p.bf16)) << 16);
                    *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(p.out) + static_cast<size_t>(trow[u]) * p.ldo + col) = o;
                }
            }
        }
    }
}

hipError_t launch_gemm_skinny(GemmDev& d, int epilogue, hipStream_t stream);
// Decode kernel (at most 64 rows per chunk): gemm_decode_plan picks the fragments per workgroup and, when
// split_max > 1, the number of K parts (the epilogue must then be EPI_PARTIAL_F32: out = fp32 [parts][M_max][ldo]).
int gemm_decode_plan(const GemmDev& d, int epilogue, int split_max, int* nwn_out);
hipError_t launch_gemm_decode(GemmDev& d, int epilogue, int nwn, int split, hipStream_t stream);
hipError_t launch_gemm_mid(GemmDev& d, int epilogue, hipStream_t stream);

}  // namespace qtale
