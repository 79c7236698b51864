// Group-wise round-to-nearest int4 quantizer and the matrix-core prepack (setup step, off the timed path).
//
// Sec. 4.1 of the paper fixes "weight-only, group size 128, 4 bit"; the arithmetic below is this
// library's reading: asymmetric min/max with zero inside the range, fp16 scale, integer zero-point,
// IEEE fp32 operations with round-half-even so that the codes are reproducible bit for bit.
#include "qtale_dev.h"
#include "qtale_kernels.h"

namespace qtale {

// One thread owns 8 consecutive k of one row (one canonical uint32 word).  The group/8 threads of a
// group are consecutive lanes of one wave and reduce min/max with xor-shuffles.
__global__ void __launch_bounds__(256)
quantize_rows_kernel(const float* __restrict__ W, int N, int K, int group, int n_groups, float qmax,
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
    if (!ok) return;
    lo = fminf(lo, 0.0f);
    hi = fmaxf(hi, 0.0f);
    const float s32 = __fdiv_rn(__fsub_rn(hi, lo), qmax);
    half_t s16 = static_cast<half_t>(s32);                                   // round to nearest even
    float sf = static_cast<float>(s16);
    if (sf == 0.0f || !(fabsf(sf) <= 65504.0f)) { s16 = static_cast<half_t>(1.0f); sf = 1.0f; }
    const float z = fminf(fmaxf(rintf(__fdiv_rn(-lo, sf)), 0.0f), qmax);
    uint32_t word = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float q = fminf(fmaxf(__fadd_rn(rintf(__fdiv_rn(v[i], sf)), z), 0.0f), qmax);
        word |= static_cast<uint32_t>(q) << (4 * i);
    }
    const int kw = (K + 7) >> 3;
    codes[static_cast<size_t>(n) * kw + w] = word;
    if ((w % wpg) == 0) {
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

PrepackDims prepack_dims(int N, int K, int group) {
    PrepackDims d;
    d.NF = (N + 31) / 32;
    d.KT = (K + 63) / 64;
    d.NGP = (d.KT * 64 + group - 1) / group;
    d.code_bytes = static_cast<size_t>(d.NF) * d.KT * 1024;
    d.sz_bytes = static_cast<size_t>(d.NGP) * d.NF * 32 * 4;
    return d;
}

hipError_t launch_quantize(const float* W, int N, int K, int bits, int group, uint32_t* codes,
                           uint16_t* scales, uint16_t* zeros, hipStream_t stream) {
    const int ng = (K + group - 1) / group;
    const long total = static_cast<long>(N) * ng * (group / 8);
    const int blocks = static_cast<int>((total + 255) / 256);
    if (blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(quantize_rows_kernel, dim3(blocks), dim3(256), 0, stream, W, N, K, group, ng,
                       static_cast<float>((1 << bits) - 1), codes, scales, zeros);
    return hipGetLastError();
}

hipError_t launch_prepack(const uint32_t* codes, const uint16_t* scales, const uint16_t* zeros, int N,
                          int K, int group, void* prepacked, hipStream_t stream) {
    const PrepackDims d = prepack_dims(N, K, group);
    const int ng = (K + group - 1) / group;
    const long n_code = static_cast<long>(d.NF) * d.KT * 64;
    const long n_sz = static_cast<long>(d.NGP) * d.NF * 32;
    const long total = n_code > n_sz ? n_code : n_sz;
    const int blocks = static_cast<int>((total + 255) / 256);
    if (blocks == 0) return hipSuccess;
    U4* pc = reinterpret_cast<U4*>(prepacked);
    uint32_t* ps = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(prepacked) + d.code_bytes);
    hipLaunchKernelGGL(prepack_kernel, dim3(blocks), dim3(256), 0, stream, codes, scales, zeros, N, K,
                       group, ng, d.NF, d.KT, d.NGP, pc, ps);
    return hipGetLastError();
}

}  // namespace qtale
