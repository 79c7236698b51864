// Group-wise round-to-nearest int4 / int3 quantizer and the matrix-core prepack (setup step, off the timed
// path).
//
// Sec. 4.1 of the paper fixes "weight-only, group size 128, 4 and 3 bit"; the arithmetic below is this
// library's reading: asymmetric min/max with zero inside the range, fp16 scale, integer zero-point,
// IEEE fp32 operations with round-half-even so that the codes are reproducible bit for bit.
#include "qtale_dev.h"
#include "qtale_kernels.h"

namespace qtale {

// One thread owns 8 consecutive k of one row (one canonical uint32 word of 4-bit codes, or 24 bits of the
// 3-bit stream).  The group/8 threads of a group are consecutive lanes of one wave and reduce min/max
// with xor-shuffles.  3-bit codes: four consecutive threads hold one 32-code block = 96 bits = 3 words of
// the row's little-endian bit stream (code k at bits 3k..3k+2); they exchange their 24-bit pieces with
// shuffles and the first three write one word each.
__global__ void __launch_bounds__(256)
quantize_rows_kernel(const float* __restrict__ W, int N, int K, int bits, int group, int n_groups, float qmax,
                     uint32_t* __restrict__ codes, uint16_t* __restrict__ scales, uint16_t* __restrict__ zeros) {
    const int wpg = group >> 3;                       // words (threads) per group: 4, 8 or 16
    const int wpr = n_groups * wpg;                   // padded words per row
    const long gid = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
    const long total = static_cast<long>(N) * wpr;
    const bool row_ok = gid < total;
    const int n = row_ok ? static_cast<int>(gid / wpr) : 0;
    const int w = row_ok ? static_cast<int>(gid % wpr) : 0;
    const int k0 = w * 8;
    const bool ok = row_ok && k0 < K;                 // K % 8 == 0, so a word is all-in or all-out

    float v[8];
    float lo = INFINITY, hi = -INFINITY;
    if (ok) {
        const float4* p = reinterpret_cast<const float4*>(W + static_cast<size_t>(n) * K + k0);
        const float4 a = p[0], b = p[1];
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
#pragma unroll
        for (int i = 0; i < 8; ++i) { lo = fminf(lo, v[i]); hi = fmaxf(hi, v[i]); }
    }
    for (int o = wpg >> 1; o > 0; o >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, o, 64));
        hi = fmaxf(hi, __shfl_xor(hi, o, 64));
    }
    lo = fminf(lo, 0.0f);
    hi = fmaxf(hi, 0.0f);
    const float s32 = __fdiv_rn(__fsub_rn(hi, lo), qmax);     // lanes outside the matrix see lo = hi = 0 here
    half_t s16 = static_cast<half_t>(s32);                                   // round to nearest even
    float sf = static_cast<float>(s16);
    if (sf == 0.0f || !(fabsf(sf) <= 65504.0f)) { s16 = static_cast<half_t>(1.0f); sf = 1.0f; }
    const float z = fminf(fmaxf(rintf(__fdiv_rn(-lo, sf)), 0.0f), qmax);
    uint32_t word = 0;
    if (ok) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float q = fminf(fmaxf(__fadd_rn(rintf(__fdiv_rn(v[i], sf)), z), 0.0f), qmax);
            word |= static_cast<uint32_t>(q) << (bits * i);
        }
    }
    if (bits == 3) {                                  // uniform branch: every lane of the wave takes part
        const int lane = threadIdx.x & 63, q0 = lane & ~3, i = lane & 3;
        const uint32_t v0 = __shfl(word, q0, 64), v1 = __shfl(word, q0 + 1, 64);
        const uint32_t v2 = __shfl(word, q0 + 2, 64), v3 = __shfl(word, q0 + 3, 64);
        const uint32_t out = i == 0 ? (v0 | (v1 << 24)) : i == 1 ? ((v1 >> 8) | (v2 << 16)) : ((v2 >> 16) | (v3 << 8));
        const int blk = w >> 2;                       // 32-code block of the row; its first thread has k0 = 32*blk
        if (row_ok && i < 3 && blk * 32 < K)
            codes[static_cast<size_t>(n) * (3 * ((K + 31) >> 5)) + 3 * blk + i] = out;
    } else if (bits == 2) {                           // two consecutive threads hold one word (16 codes)
        const int lane = threadIdx.x & 63;
        const uint32_t lo16 = __shfl(word, lane & ~1, 64), hi16 = __shfl(word, lane | 1, 64);
        if (ok && (lane & 1) == 0) codes[static_cast<size_t>(n) * ((K + 15) >> 4) + (w >> 1)] = lo16 | (hi16 << 16);
    } else if (ok) {
        codes[static_cast<size_t>(n) * ((K + 7) >> 3) + w] = word;
    }
    if (ok && (w % wpg) == 0) {
        const int g = w / wpg;
        scales[static_cast<size_t>(n) * n_groups + g] = __builtin_bit_cast(uint16_t, s16);
        zeros[static_cast<size_t>(n) * n_groups + g] = __builtin_bit_cast(uint16_t, static_cast<half_t>(z));
    }
}

// Prepacked layout read by the GEMM kernels.
//   codes: [NF][KT][64 lanes] x 16 bytes.  NF = ceil(N/32) row fragments, KT = ceil(K/64) k-tiles.
//          Lane l of fragment f, k-tile kt holds, in 32-bit word j (0..3), the eight codes of row
//          n = 32 f + l%32 for k = 64 kt + 16 j + 8 (l/32) + e, e = 0..7, with code e stored at bit
//          4*(e/2) + 16*(e%2): masking with 0x000f000f / 0x00f000f0 on the word and on word>>8 yields
//          the fp16 pairs (e0,e1), (e2,e3), (e4,e5), (e6,e7) directly.
//          Rows n >= N get scale 0; positions k >= K get the group's zero-point (dequantize to 0).
//   sz:    [NGP][NF*32] x 4 bytes: fp16 scale in the low half, fp16 zero-point in the high half,
//          NGP = ceil(KT*64/group) groups.
__global__ void __launch_bounds__(256)
prepack_kernel(const uint32_t* __restrict__ codes, const uint16_t* __restrict__ scales,
               const uint16_t* __restrict__ zeros, int N, int K, int group, int n_groups,
               int NF, int KT, int NGP, U4* __restrict__ pcodes, uint32_t* __restrict__ psz) {
    const long gid = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
    const long n_code = static_cast<long>(NF) * KT * 64;
    const int kw = (K + 7) >> 3;
    if (gid < n_code) {
        const int lane = static_cast<int>(gid & 63);
        const long t = gid >> 6;
        const int kt = static_cast<int>(t % KT);
        const int f = static_cast<int>(t / KT);
        const int n = f * 32 + (lane & 31);
        uint32_t out[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int k0 = kt * 64 + j * 16 + (lane >> 5) * 8;
            uint32_t src = 0;
            if (n < N) {
                if (k0 < K) {
                    src = codes[static_cast<size_t>(n) * kw + (k0 >> 3)];
                } else {
                    const int g = k0 / group;
                    const uint32_t zc = g < n_groups
                        ? static_cast<uint32_t>(static_cast<float>(__builtin_bit_cast(half_t, zeros[static_cast<size_t>(n) * n_groups + g])))
                        : 0u;
                    src = zc * 0x11111111u;
                }
            }
            uint32_t w = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t c = (src >> (4 * e)) & 0xFu;
                w |= c << (4 * (e >> 1) + 16 * (e & 1));
            }
            out[j] = w;
        }
        pcodes[gid] = U4{out[0], out[1], out[2], out[3]};
    }
    const long n_sz = static_cast<long>(NGP) * NF * 32;
    if (gid < n_sz) {
        const int n = static_cast<int>(gid % (NF * 32));
        const int g = static_cast<int>(gid / (NF * 32));
        uint32_t v = 0;
        if (n < N && g < n_groups) {
            v = static_cast<uint32_t>(scales[static_cast<size_t>(n) * n_groups + g]) |
                (static_cast<uint32_t>(zeros[static_cast<size_t>(n) * n_groups + g]) << 16);
        }
        psz[gid] = v;
    }
}

// 3-bit codes.  Same fragment / k-tile order, 12 bytes per lane: the lane's 32 codes q = 8 j + e (k-step j,
// element e, k = 64 kt + 16 j + 8 (l/32) + e) form 16 pairs h = q/2; pair h < 15 sits in word h/5 at bit
// 3*(h%5) of the low half (even code) and of the high half (odd code); pair 15 is spread over the spare
// bits 15 (even code) and 31 (odd code) of the three words, bit i of the code in word i.  sz as above.
__global__ void __launch_bounds__(256)
prepack3_kernel(const uint32_t* __restrict__ codes, const uint16_t* __restrict__ scales,
                const uint16_t* __restrict__ zeros, int N, int K, int group, int n_groups,
                int NF, int KT, int NGP, uint32_t* __restrict__ pcodes, uint32_t* __restrict__ psz) {
    const long gid = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
    const long n_code = static_cast<long>(NF) * KT * 64;
    const int kw = 3 * ((K + 31) >> 5);
    if (gid < n_code) {
        const int lane = static_cast<int>(gid & 63);
        const long t = gid >> 6;
        const int kt = static_cast<int>(t % KT);
        const int f = static_cast<int>(t / KT);
        const int n = f * 32 + (lane & 31);
        uint32_t out[3] = {0u, 0u, 0u};
        for (int q = 0; q < 32; ++q) {
            const int k = kt * 64 + (q >> 3) * 16 + (lane >> 5) * 8 + (q & 7);
            uint32_t c = 0;
            if (n < N) {
                if (k < K) {
                    const uint32_t* row = codes + static_cast<size_t>(n) * kw;
                    const int bit = 3 * k, wi = bit >> 5, off = bit & 31;
                    uint32_t v = row[wi] >> off;
                    if (off > 29) v |= row[wi + 1] << (32 - off);
                    c = v & 7u;
                } else {
                    const int g = k / group;
                    c = g < n_groups
                        ? static_cast<uint32_t>(static_cast<float>(__builtin_bit_cast(half_t, zeros[static_cast<size_t>(n) * n_groups + g])))
                        : 0u;
                }
            }
            const int h = q >> 1, hs = (q & 1) * 16;
            if (h < 15) {
                out[h / 5] |= c << (3 * (h % 5) + hs);
            } else {
                out[0] |= (c & 1u) << (15 + hs);
                out[1] |= ((c >> 1) & 1u) << (15 + hs);
                out[2] |= ((c >> 2) & 1u) << (15 + hs);
            }
        }
        pcodes[gid * 3 + 0] = out[0];
        pcodes[gid * 3 + 1] = out[1];
        pcodes[gid * 3 + 2] = out[2];
    }
    const long n_sz = static_cast<long>(NGP) * NF * 32;
    if (gid < n_sz) {
        const int n = static_cast<int>(gid % (NF * 32));
        const int g = static_cast<int>(gid / (NF * 32));
        uint32_t v = 0;
        if (n < N && g < n_groups) {
            v = static_cast<uint32_t>(scales[static_cast<size_t>(n) * n_groups + g]) |
                (static_cast<uint32_t>(zeros[static_cast<size_t>(n) * n_groups + g]) << 16);
        }
        psz[gid] = v;
    }
}

// 2-bit codes.  Same fragment / k-tile order, 8 bytes per lane: pair h = q/2 of the lane's 32 codes sits in word
// h/8 at bit 2*(h%8) of the low half (even code) and of the high half (odd code).  sz as above.
__global__ void __launch_bounds__(256)
prepack2_kernel(const uint32_t* __restrict__ codes, const uint16_t* __restrict__ scales,
                const uint16_t* __restrict__ zeros, int N, int K, int group, int n_groups,
                int NF, int KT, int NGP, uint32_t* __restrict__ pcodes, uint32_t* __restrict__ psz) {
    const long gid = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
    const long n_code = static_cast<long>(NF) * KT * 64;
    const int kw = (K + 15) >> 4;
    if (gid < n_code) {
        const int lane = static_cast<int>(gid & 63);
        const long t = gid >> 6;
        const int kt = static_cast<int>(t % KT);
        const int f = static_cast<int>(t / KT);
        const int n = f * 32 + (lane & 31);
        uint32_t out[2] = {0u, 0u};
        for (int q = 0; q < 32; ++q) {
            const int k = kt * 64 + (q >> 3) * 16 + (lane >> 5) * 8 + (q & 7);
            uint32_t c = 0;
            if (n < N) {
                if (k < K) {
                    c = (codes[static_cast<size_t>(n) * kw + (k >> 4)] >> (2 * (k & 15))) & 3u;
                } else {
                    const int g = k / group;
                    c = g < n_groups
                        ? static_cast<uint32_t>(static_cast<float>(__builtin_bit_cast(half_t, zeros[static_cast<size_t>(n) * n_groups + g])))
                        : 0u;
                }
            }
            const int h = q >> 1;
            out[h >> 3] |= c << (2 * (h & 7) + (q & 1) * 16);
        }
        pcodes[gid * 2 + 0] = out[0];
        pcodes[gid * 2 + 1] = out[1];
    }
    const long n_sz = static_cast<long>(NGP) * NF * 32;
    if (gid < n_sz) {
        const int n = static_cast<int>(gid % (NF * 32));
        const int g = static_cast<int>(gid / (NF * 32));
        uint32_t v = 0;
        if (n < N && g < n_groups) {
            v = static_cast<uint32_t>(scales[static_cast<size_t>(n) * n_groups + g]) |
                (static_cast<uint32_t>(zeros[static_cast<size_t>(n) * n_groups + g]) << 16);
        }
        psz[gid] = v;
    }
}

PrepackDims prepack_dims(int N, int K, int group, int bits) {
    PrepackDims d;
    d.NF = (N + 31) / 32;
    d.KT = (K + 63) / 64;
    d.NGP = (d.KT * 64 + group - 1) / group;
    d.code_bytes = static_cast<size_t>(d.NF) * d.KT * (bits == 3 ? 768 : bits == 2 ? 512 : 1024);
    d.sz_bytes = static_cast<size_t>(d.NGP) * d.NF * 32 * 4;
    return d;
}

hipError_t launch_quantize(const float* W, int N, int K, int bits, int group, uint32_t* codes,
                           uint16_t* scales, uint16_t* zeros, hipStream_t stream) {
    const int ng = (K + group - 1) / group;
    const long total = static_cast<long>(N) * ng * (group / 8);
    const int blocks = static_cast<int>((total + 255) / 256);
    if (blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(quantize_rows_kernel, dim3(blocks), dim3(256), 0, stream, W, N, K, bits, group, ng,
                       static_cast<float>((1 << bits) - 1), codes, scales, zeros);
    return hipGetLastError();
}

hipError_t launch_prepack(const uint32_t* codes, const uint16_t* scales, const uint16_t* zeros, int N,
                          int K, int bits, int group, void* prepacked, hipStream_t stream) {
    const PrepackDims d = prepack_dims(N, K, group, bits);
    const int ng = (K + group - 1) / group;
    const long n_code = static_cast<long>(d.NF) * d.KT * 64;
    const long n_sz = static_cast<long>(d.NGP) * d.NF * 32;
    const long total = n_code > n_sz ? n_code : n_sz;
    const int blocks = static_cast<int>((total + 255) / 256);
    if (blocks == 0) return hipSuccess;
    U4* pc = reinterpret_cast<U4*>(prepacked);
    uint32_t* ps = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(prepacked) + d.code_bytes);
    if (bits == 2) {
        hipLaunchKernelGGL(prepack2_kernel, dim3(blocks), dim3(256), 0, stream, codes, scales, zeros, N, K,
                           group, ng, d.NF, d.KT, d.NGP, reinterpret_cast<uint32_t*>(prepacked), ps);
        return hipGetLastError();
    }
    if (bits == 3) {
        hipLaunchKernelGGL(prepack3_kernel, dim3(blocks), dim3(256), 0, stream, codes, scales, zeros, N, K,
                           group, ng, d.NF, d.KT, d.NGP, reinterpret_cast<uint32_t*>(prepacked), ps);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(prepack_kernel, dim3(blocks), dim3(256), 0, stream, codes, scales, zeros, N, K,
                       group, ng, d.NF, d.KT, d.NGP, pc, ps);
    return hipGetLastError();
}

}  // namespace qtale
