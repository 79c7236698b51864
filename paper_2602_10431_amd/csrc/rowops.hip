// Row-wise kernels on the compacted (executed) tokens: gather + RMSNorm, RMSNorm of the fp32 residual,
// rotary embedding at the token's original position with optional K/V cache append.
// All are bandwidth-bound: 16-byte loads, one wave per row, fp32 reductions.
#include "qtale_dev.h"
#include "qtale_kernels.h"

namespace qtale {

// out[i] = fp16( x[idx[i]] / sqrt(mean(x^2) + eps) * gain ), one wave per executed row (App. B.2 gather
// fused with the layer's first normalisation).
template <bool BF16>
__global__ void __launch_bounds__(256)
gather_rmsnorm_kernel(const uint16_t* __restrict__ x, int H, const int32_t* __restrict__ idx,
                      const int32_t* __restrict__ count, const uint16_t* __restrict__ gain, float eps,
                      uint16_t* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= *count) return;
    const int t = idx[i];
    const U4* xr = reinterpret_cast<const U4*>(x + static_cast<size_t>(t) * H);
    const U4* gr = reinterpret_cast<const U4*>(gain);
    U4* orow = reinterpret_cast<U4*>(out + static_cast<size_t>(i) * H);
    const int chunks = H >> 3;
    float ss = 0.0f;
    for (int c = lane; c < chunks; c += 64) {
        const U4 v = xr[c];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float a = act_to_float<BF16>(static_cast<uint16_t>(w[j] & 0xffffu));
            const float b = act_to_float<BF16>(static_cast<uint16_t>(w[j] >> 16));
            ss = fmaf(a, a, ss);
            ss = fmaf(b, b, ss);
        }
    }
    ss = wave_sum(ss);
    const float inv = 1.0f / sqrtf(ss / static_cast<float>(H) + eps);
    for (int c = lane; c < chunks; c += 64) {
        const U4 v = xr[c];
        const U4 g = gr[c];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        const uint32_t gw[4] = {g.x, g.y, g.z, g.w};
        uint32_t o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float a = act_to_float<BF16>(static_cast<uint16_t>(w[j] & 0xffffu)) * inv *
                            act_to_float<BF16>(static_cast<uint16_t>(gw[j] & 0xffffu));
            const float b = act_to_float<BF16>(static_cast<uint16_t>(w[j] >> 16)) * inv *
                            act_to_float<BF16>(static_cast<uint16_t>(gw[j] >> 16));
            o[j] = static_cast<uint32_t>(float_to_half_bits(a)) | (static_cast<uint32_t>(float_to_half_bits(b)) << 16);
        }
        orow[c] = U4{o[0], o[1], o[2], o[3]};
    }
}

hipError_t launch_gather_rmsnorm(const void* x, int bf16, int H, const int32_t* idx, const int32_t* count,
                                 int max_rows, const void* gain, float eps, void* out_f16, hipStream_t stream) {
    if (max_rows == 0) return hipSuccess;
    const dim3 grid((max_rows + 3) / 4), block(256);
    if (bf16)
        hipLaunchKernelGGL(gather_rmsnorm_kernel<true>, grid, block, 0, stream, reinterpret_cast<const uint16_t*>(x),
                           H, idx, count, reinterpret_cast<const uint16_t*>(gain), eps, reinterpret_cast<uint16_t*>(out_f16));
    else
        hipLaunchKernelGGL(gather_rmsnorm_kernel<false>, grid, block, 0, stream, reinterpret_cast<const uint16_t*>(x),
                           H, idx, count, reinterpret_cast<const uint16_t*>(gain), eps, reinterpret_cast<uint16_t*>(out_f16));
    return hipGetLastError();
}

// out[i] = fp16( h[i] / sqrt(mean(h^2) + eps) * gain ) for the fp32 post-attention residual h.
template <bool BF16>
__global__ void __launch_bounds__(256)
rmsnorm_f32_kernel(const float* __restrict__ h, int H, const int32_t* __restrict__ count,
                   const uint16_t* __restrict__ gain, float eps, uint16_t* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= *count) return;
    const float4* hr = reinterpret_cast<const float4*>(h + static_cast<size_t>(i) * H);
    const U2* gr = reinterpret_cast<const U2*>(gain);
    U2* orow = reinterpret_cast<U2*>(out + static_cast<size_t>(i) * H);
    const int chunks = H >> 2;
    float ss = 0.0f;
    for (int c = lane; c < chunks; c += 64) {
        const float4 v = hr[c];
        ss = fmaf(v.x, v.x, ss); ss = fmaf(v.y, v.y, ss); ss = fmaf(v.z, v.z, ss); ss = fmaf(v.w, v.w, ss);
    }
    ss = wave_sum(ss);
    const float inv = 1.0f / sqrtf(ss / static_cast<float>(H) + eps);
    for (int c = lane; c < chunks; c += 64) {
        const float4 v = hr[c];
        const U2 g = gr[c];
        const float g0 = act_to_float<BF16>(static_cast<uint16_t>(g.x & 0xffffu));
        const float g1 = act_to_float<BF16>(static_cast<uint16_t>(g.x >> 16));
        const float g2 = act_to_float<BF16>(static_cast<uint16_t>(g.y & 0xffffu));
        const float g3 = act_to_float<BF16>(static_cast<uint16_t>(g.y >> 16));
        U2 o;
        o.x = static_cast<uint32_t>(float_to_half_bits(v.x * inv * g0)) | (static_cast<uint32_t>(float_to_half_bits(v.y * inv * g1)) << 16);
        o.y = static_cast<uint32_t>(float_to_half_bits(v.z * inv * g2)) | (static_cast<uint32_t>(float_to_half_bits(v.w * inv * g3)) << 16);
        orow[c] = o;
    }
}

hipError_t launch_rmsnorm_f32(const float* h, int H, const int32_t* count, int max_rows, const void* gain,
                              int gain_bf16, float eps, void* out_f16, hipStream_t stream) {
    if (max_rows == 0) return hipSuccess;
    const dim3 grid((max_rows + 3) / 4), block(256);
    if (gain_bf16)
        hipLaunchKernelGGL(rmsnorm_f32_kernel<true>, grid, block, 0, stream, h, H, count,
                           reinterpret_cast<const uint16_t*>(gain), eps, reinterpret_cast<uint16_t*>(out_f16));
    else
        hipLaunchKernelGGL(rmsnorm_f32_kernel<false>, grid, block, 0, stream, h, H, count,
                           reinterpret_cast<const uint16_t*>(gain), eps, reinterpret_cast<uint16_t*>(out_f16));
    return hipGetLastError();
}

// Rotary embedding, half-split pairing (element i with i + d/2), angle = position * base^(-2i/d), at
// the ORIGINAL absolute position of the token (a bypassed token leaves a gap in the positions seen by
// a layer).  One workgroup per executed row: the d/2 (cos, sin) pairs of the row's position are
// evaluated once in fp64 into LDS, then every thread rotates 8 pairs of one q or k head with 16-byte
// accesses.  With a cache, rotated k and v are also appended at kv_old[seq] + (rank of the row inside
// its sequence).
__global__ void __launch_bounds__(256)
rope_append_kernel(RopeArgs a) {
    __shared__ float cs[64], sn[64];              // head_dim <= 128
    const int i = blockIdx.x;
    if (i >= *a.count) return;
    const int t = a.idx[i];
    const int d = a.d, half = d >> 1;
    const int width = (a.nh + 2 * a.nkv) * d;
    half_t* row = reinterpret_cast<half_t*>(a.qkv) + static_cast<size_t>(i) * width;
    half_t* kdst = nullptr;
    half_t* vdst = nullptr;
    if (a.k_cache) {
        const int b = a.row_seq[i];
        const int slot = a.kv_old[b] + (i - a.cu_exec[b]);
        if (slot < a.cap) {
            const size_t off = (static_cast<size_t>(b) * a.cap + slot) * (static_cast<size_t>(a.nkv) * d);
            kdst = reinterpret_cast<half_t*>(a.k_cache) + off;
            vdst = reinterpret_cast<half_t*>(a.v_cache) + off;
        }
    }
    if (threadIdx.x < half) {
        const int p = threadIdx.x;
        const double inv_freq = pow(static_cast<double>(a.base), -2.0 * static_cast<double>(p) / static_cast<double>(d));
        double s, c;
        sincos(static_cast<double>(a.positions[t]) * inv_freq, &s, &c);
        cs[p] = static_cast<float>(c);
        sn[p] = static_cast<float>(s);
    }
    __syncthreads();
    const int cph = half >> 3;                     // 8-pair chunks per head
    const int items = (a.nh + a.nkv) * cph;
    for (int w = threadIdx.x; w < items; w += blockDim.x) {
        const int hd = w / cph, p0 = (w % cph) * 8;
        half_t* hp = row + static_cast<size_t>(hd) * d;
        const half8_t lo = *reinterpret_cast<const half8_t*>(hp + p0);
        const half8_t hi = *reinterpret_cast<const half8_t*>(hp + p0 + half);
        half8_t rlo, rhi;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float l = static_cast<float>(lo[e]), h = static_cast<float>(hi[e]);
            const float c = cs[p0 + e], s = sn[p0 + e];
            rlo[e] = static_cast<half_t>(l * c - h * s);
            rhi[e] = static_cast<half_t>(h * c + l * s);
        }
        *reinterpret_cast<half8_t*>(hp + p0) = rlo;
        *reinterpret_cast<half8_t*>(hp + p0 + half) = rhi;
        if (kdst && hd >= a.nh) {
            *reinterpret_cast<half8_t*>(kdst + (hd - a.nh) * d + p0) = rlo;
            *reinterpret_cast<half8_t*>(kdst + (hd - a.nh) * d + p0 + half) = rhi;
        }
    }
    if (vdst) {
        const half8_t* vsrc = reinterpret_cast<const half8_t*>(row + static_cast<size_t>(a.nh + a.nkv) * d);
        for (int e = threadIdx.x; e < (a.nkv * d) >> 3; e += blockDim.x) reinterpret_cast<half8_t*>(vdst)[e] = vsrc[e];
    }
}

hipError_t launch_rope_append(const RopeArgs& a, hipStream_t stream) {
    if (a.max_rows == 0) return hipSuccess;
    hipLaunchKernelGGL(rope_append_kernel, dim3(a.max_rows), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace qtale
