// Row-wise kernels on the compacted (executed) tokens: gather + RMSNorm, RMSNorm of the fp32 residual,
// rotary embedding at the token's original position with optional K/V cache append.
// All are bandwidth-bound: 16-byte loads, one workgroup per row, fp32 reductions.
#include "qtale_dev.h"
#include "qtale_kernels.h"

namespace qtale {

// Sum over the 256 threads of a workgroup (4 waves), result in every thread.
__device__ __forceinline__ float block_sum_256(float v, float* red) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

// out[i] = fp16( x[idx[i]] / sqrt(mean(x^2) + eps) * gain ), one workgroup per executed row (App. B.2
// gather fused with the layer's first normalisation).  A thread keeps its 8-element chunks in registers
// between the reduction and the scaling (up to 8192 columns; wider rows re-read from L2).
template <bool BF16>
__global__ void __launch_bounds__(256)
gather_rmsnorm_kernel(const uint16_t* __restrict__ x, int H, const int32_t* __restrict__ idx,
                      const int32_t* __restrict__ count, const uint16_t* __restrict__ gain, float eps,
                      uint16_t* __restrict__ out) {
    __shared__ float red[4];
    const int i = blockIdx.x;
    if (i >= *count) return;
    const int t = idx[i];
    const u32x4_t* xr = reinterpret_cast<const u32x4_t*>(x + static_cast<size_t>(t) * H);
    const u32x4_t* gr = reinterpret_cast<const u32x4_t*>(gain);
    u32x4_t* orow = reinterpret_cast<u32x4_t*>(out + static_cast<size_t>(i) * H);
    const int chunks = H >> 3;
    constexpr int KEEP = 4;
    u32x4_t keep[KEEP];
    float ss = 0.0f;
#pragma unroll
    for (int u = 0; u < KEEP; ++u) {
        const int c = threadIdx.x + u * 256;
        keep[u] = c < chunks ? xr[c] : u32x4_t{0u, 0u, 0u, 0u};
    }
    auto sumsq = [&](const u32x4_t& v) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float a = act_to_float<BF16>(static_cast<uint16_t>(v[j] & 0xffffu));
            const float b = act_to_float<BF16>(static_cast<uint16_t>(v[j] >> 16));
            ss = fmaf(a, a, ss);
            ss = fmaf(b, b, ss);
        }
    };
#pragma unroll
    for (int u = 0; u < KEEP; ++u) sumsq(keep[u]);
    for (int c = threadIdx.x + KEEP * 256; c < chunks; c += 256) sumsq(xr[c]);
    ss = block_sum_256(ss, red);
    const float inv = 1.0f / sqrtf(ss / static_cast<float>(H) + eps);
    auto emit = [&](int c, const u32x4_t& v) {
        const u32x4_t g = gr[c];
        u32x4_t o;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float a = act_to_float<BF16>(static_cast<uint16_t>(v[j] & 0xffffu)) * inv *
                            act_to_float<BF16>(static_cast<uint16_t>(g[j] & 0xffffu));
            const float b = act_to_float<BF16>(static_cast<uint16_t>(v[j] >> 16)) * inv *
                            act_to_float<BF16>(static_cast<uint16_t>(g[j] >> 16));
            o[j] = static_cast<uint32_t>(float_to_half_bits(a)) | (static_cast<uint32_t>(float_to_half_bits(b)) << 16);
        }
        orow[c] = o;
    };
#pragma unroll
    for (int u = 0; u < KEEP; ++u) {
        const int c = threadIdx.x + u * 256;
        if (c < chunks) emit(c, keep[u]);
    }
    for (int c = threadIdx.x + KEEP * 256; c < chunks; c += 256) emit(c, xr[c]);
}

hipError_t launch_gather_rmsnorm(const void* x, int bf16, int H, const int32_t* idx, const int32_t* count,
                                 int max_rows, const void* gain, float eps, void* out_f16, hipStream_t stream) {
    if (max_rows == 0) return hipSuccess;
    const dim3 grid(max_rows), block(256);
    if (bf16)
        hipLaunchKernelGGL(gather_rmsnorm_kernel<true>, grid, block, 0, stream, reinterpret_cast<const uint16_t*>(x),
                           H, idx, count, reinterpret_cast<const uint16_t*>(gain), eps, reinterpret_cast<uint16_t*>(out_f16));
    else
        hipLaunchKernelGGL(gather_rmsnorm_kernel<false>, grid, block, 0, stream, reinterpret_cast<const uint16_t*>(x),
                           H, idx, count, reinterpret_cast<const uint16_t*>(gain), eps, reinterpret_cast<uint16_t*>(out_f16));
    return hipGetLastError();
}

// out[i] = fp16( h[i] / sqrt(mean(h^2) + eps) * gain ) for the fp32 post-attention residual h; one
// workgroup per row, the row held in registers between the two steps (up to 8192 columns).
template <bool BF16>
__global__ void __launch_bounds__(256)
rmsnorm_f32_kernel(const float* __restrict__ h, int H, const int32_t* __restrict__ count,
                   const uint16_t* __restrict__ gain, float eps, uint16_t* __restrict__ out) {
    __shared__ float red[4];
    const int i = blockIdx.x;
    if (i >= *count) return;
    const float4_t* hr = reinterpret_cast<const float4_t*>(h + static_cast<size_t>(i) * H);
    const U2* gr = reinterpret_cast<const U2*>(gain);
    U2* orow = reinterpret_cast<U2*>(out + static_cast<size_t>(i) * H);
    const int chunks = H >> 2;
    constexpr int KEEP = 8;
    float4_t keep[KEEP];
    float ss = 0.0f;
#pragma unroll
    for (int u = 0; u < KEEP; ++u) {
        const int c = threadIdx.x + u * 256;
        keep[u] = c < chunks ? hr[c] : float4_t{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int u = 0; u < KEEP; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e) ss = fmaf(keep[u][e], keep[u][e], ss);
    for (int c = threadIdx.x + KEEP * 256; c < chunks; c += 256) {
        const float4_t v = hr[c];
#pragma unroll
        for (int e = 0; e < 4; ++e) ss = fmaf(v[e], v[e], ss);
    }
    ss = block_sum_256(ss, red);
    const float inv = 1.0f / sqrtf(ss / static_cast<float>(H) + eps);
    auto emit = [&](int c, const float4_t& v) {
        const U2 g = gr[c];
        const float g0 = act_to_float<BF16>(static_cast<uint16_t>(g.x & 0xffffu));
        const float g1 = act_to_float<BF16>(static_cast<uint16_t>(g.x >> 16));
        const float g2 = act_to_float<BF16>(static_cast<uint16_t>(g.y & 0xffffu));
        const float g3 = act_to_float<BF16>(static_cast<uint16_t>(g.y >> 16));
        U2 o;
        o.x = static_cast<uint32_t>(float_to_half_bits(v[0] * inv * g0)) | (static_cast<uint32_t>(float_to_half_bits(v[1] * inv * g1)) << 16);
        o.y = static_cast<uint32_t>(float_to_half_bits(v[2] * inv * g2)) | (static_cast<uint32_t>(float_to_half_bits(v[3] * inv * g3)) << 16);
        orow[c] = o;
    };
#pragma unroll
    for (int u = 0; u < KEEP; ++u) {
        const int c = threadIdx.x + u * 256;
        if (c < chunks) emit(c, keep[u]);
    }
    for (int c = threadIdx.x + KEEP * 256; c < chunks; c += 256) emit(c, hr[c]);
}

hipError_t launch_rmsnorm_f32(const float* h, int H, const int32_t* count, int max_rows, const void* gain,
                              int gain_bf16, float eps, void* out_f16, hipStream_t stream) {
    if (max_rows == 0) return hipSuccess;
    const dim3 grid(max_rows), block(256);
    if (gain_bf16)
        hipLaunchKernelGGL(rmsnorm_f32_kernel<true>, grid, block, 0, stream, h, H, count,
                           reinterpret_cast<const uint16_t*>(gain), eps, reinterpret_cast<uint16_t*>(out_f16));
    else
        hipLaunchKernelGGL(rmsnorm_f32_kernel<false>, grid, block, 0, stream, h, H, count,
                           reinterpret_cast<const uint16_t*>(gain), eps, reinterpret_cast<uint16_t*>(out_f16));
    return hipGetLastError();
}

// Consumers of the decode GEMM's fp32 partial tiles (part[s][i][c], s = K part): the parts of a row are added
// in part order, so the result does not depend on scheduling.
//   h[i] = x[idx[i]] + sum_s part[s][i]   (post-attention residual, fp32)   and   out[i] = fp16(rmsnorm(h[i]) * gain)
// One workgroup per executed row; the row stays in registers between the reduction and the scaling (up to 8192
// columns; wider rows are recomputed from the stored h).
template <bool BF16>
__global__ void __launch_bounds__(256)
reduce_rmsnorm_kernel(const float* __restrict__ part, int n_parts, size_t part_stride, const uint16_t* __restrict__ x,
                      const int32_t* __restrict__ idx, int H, const int32_t* __restrict__ count,
                      const uint16_t* __restrict__ gain, float eps, float* __restrict__ h, uint16_t* __restrict__ out) {
    __shared__ float red[4];
    const int i = blockIdx.x;
    if (i >= *count) return;
    const U2* xr = reinterpret_cast<const U2*>(x + static_cast<size_t>(idx[i]) * H);
    const float4_t* pr = reinterpret_cast<const float4_t*>(part + static_cast<size_t>(i) * H);
    const size_t pstep = part_stride / 4;
    float4_t* hr = reinterpret_cast<float4_t*>(h + static_cast<size_t>(i) * H);
    const U2* gr = reinterpret_cast<const U2*>(gain);
    U2* orow = reinterpret_cast<U2*>(out + static_cast<size_t>(i) * H);
    const int chunks = H >> 2;
    constexpr int KEEP = 8;
    float4_t keep[KEEP];
    float ss = 0.0f;
    auto row_value = [&](int c) {
        const U2 xv = xr[c];
        float4_t v;
        v[0] = act_to_float<BF16>(static_cast<uint16_t>(xv.x & 0xffffu));
        v[1] = act_to_float<BF16>(static_cast<uint16_t>(xv.x >> 16));
        v[2] = act_to_float<BF16>(static_cast<uint16_t>(xv.y & 0xffffu));
        v[3] = act_to_float<BF16>(static_cast<uint16_t>(xv.y >> 16));
        // all parts are requested before any is added (independent loads); parts past n_parts repeat part 0, unused
        float4_t pv[kGemmPartMax];
#pragma unroll
        for (int s = 0; s < kGemmPartMax; ++s) pv[s] = pr[(s < n_parts ? s : 0) * pstep + c];
        float4_t acc = pv[0];
#pragma unroll
        for (int s = 1; s < kGemmPartMax; ++s)
            if (s < n_parts) acc += pv[s];
        return v + acc;
    };
#pragma unroll
    for (int u = 0; u < KEEP; ++u) {
        const int c = threadIdx.x + u * 256;
        keep[u] = float4_t{0.f, 0.f, 0.f, 0.f};
        if (c < chunks) {
            keep[u] = row_value(c);
            hr[c] = keep[u];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) ss = fmaf(keep[u][e], keep[u][e], ss);
    }
    for (int c = threadIdx.x + KEEP * 256; c < chunks; c += 256) {
        const float4_t v = row_value(c);
        hr[c] = v;
#pragma unroll
        for (int e = 0; e < 4; ++e) ss = fmaf(v[e], v[e], ss);
    }
    ss = block_sum_256(ss, red);
    const float inv = 1.0f / sqrtf(ss / static_cast<float>(H) + eps);
    auto emit = [&](int c, const float4_t& v) {
        const U2 g = gr[c];
        const float g0 = act_to_float<BF16>(static_cast<uint16_t>(g.x & 0xffffu));
        const float g1 = act_to_float<BF16>(static_cast<uint16_t>(g.x >> 16));
        const float g2 = act_to_float<BF16>(static_cast<uint16_t>(g.y & 0xffffu));
        const float g3 = act_to_float<BF16>(static_cast<uint16_t>(g.y >> 16));
        U2 o;
        o.x = static_cast<uint32_t>(float_to_half_bits(v[0] * inv * g0)) | (static_cast<uint32_t>(float_to_half_bits(v[1] * inv * g1)) << 16);
        o.y = static_cast<uint32_t>(float_to_half_bits(v[2] * inv * g2)) | (static_cast<uint32_t>(float_to_half_bits(v[3] * inv * g3)) << 16);
        orow[c] = o;
    };
#pragma unroll
    for (int u = 0; u < KEEP; ++u) {
        const int c = threadIdx.x + u * 256;
        if (c < chunks) emit(c, keep[u]);
    }
    for (int c = threadIdx.x + KEEP * 256; c < chunks; c += 256) emit(c, row_value(c));
}

hipError_t launch_reduce_rmsnorm(const float* part, int n_parts, const void* x, int bf16, const int32_t* idx, int H,
                                 const int32_t* count, int max_rows, const void* gain, float eps, float* h,
                                 void* out_f16, hipStream_t stream) {
    if (max_rows == 0) return hipSuccess;
    const dim3 grid(max_rows), block(256);
    const size_t stride = static_cast<size_t>(max_rows) * H;
    if (bf16)
        hipLaunchKernelGGL(reduce_rmsnorm_kernel<true>, grid, block, 0, stream, part, n_parts, stride,
                           reinterpret_cast<const uint16_t*>(x), idx, H, count, reinterpret_cast<const uint16_t*>(gain), eps, h,
                           reinterpret_cast<uint16_t*>(out_f16));
    else
        hipLaunchKernelGGL(reduce_rmsnorm_kernel<false>, grid, block, 0, stream, part, n_parts, stride,
                           reinterpret_cast<const uint16_t*>(x), idx, H, count, reinterpret_cast<const uint16_t*>(gain), eps, h,
                           reinterpret_cast<uint16_t*>(out_f16));
    return hipGetLastError();
}

//   x[idx[i]] = act dtype( h[i] + sum_s part[s][i] ): the layer's output rows written back into the residual stream
// (Eq. 1 for executed tokens; bypassed rows are not touched, Eq. 3).  A row is cut over gridDim.y workgroups.
template <bool BF16>
__global__ void __launch_bounds__(256)
reduce_scatter_kernel(const float* __restrict__ part, int n_parts, size_t part_stride, const float* __restrict__ h, int H,
                      const int32_t* __restrict__ idx, const int32_t* __restrict__ count, uint16_t* __restrict__ x) {
    const int i = blockIdx.x;
    if (i >= *count) return;
    const float4_t* pr = reinterpret_cast<const float4_t*>(part + static_cast<size_t>(i) * H);
    const size_t pstep = part_stride / 4;
    const float4_t* hr = reinterpret_cast<const float4_t*>(h + static_cast<size_t>(i) * H);
    U2* orow = reinterpret_cast<U2*>(x + static_cast<size_t>(idx[i]) * H);
    const int chunks = H >> 2;
    for (int c = blockIdx.y * 256 + threadIdx.x; c < chunks; c += 256 * gridDim.y) {
        float4_t pv[kGemmPartMax];
#pragma unroll
        for (int s = 0; s < kGemmPartMax; ++s) pv[s] = pr[(s < n_parts ? s : 0) * pstep + c];
        float4_t acc = pv[0];
#pragma unroll
        for (int s = 1; s < kGemmPartMax; ++s)
            if (s < n_parts) acc += pv[s];
        const float4_t v = hr[c] + acc;
        U2 o;
        o.x = static_cast<uint32_t>(float_to_act<BF16>(v[0])) | (static_cast<uint32_t>(float_to_act<BF16>(v[1])) << 16);
        o.y = static_cast<uint32_t>(float_to_act<BF16>(v[2])) | (static_cast<uint32_t>(float_to_act<BF16>(v[3])) << 16);
        orow[c] = o;
    }
}

hipError_t launch_reduce_scatter(const float* part, int n_parts, const float* h, int H, const int32_t* idx,
                                 const int32_t* count, int max_rows, void* x, int bf16, hipStream_t stream) {
    if (max_rows == 0) return hipSuccess;
    const dim3 grid(max_rows, (H / 4 + 255) / 256), block(256);     // one 16-byte chunk per thread
    const size_t stride = static_cast<size_t>(max_rows) * H;
    if (bf16)
        hipLaunchKernelGGL(reduce_scatter_kernel<true>, grid, block, 0, stream, part, n_parts, stride, h, H, idx, count,
                           reinterpret_cast<uint16_t*>(x));
    else
        hipLaunchKernelGGL(reduce_scatter_kernel<false>, grid, block, 0, stream, part, n_parts, stride, h, H, idx, count,
                           reinterpret_cast<uint16_t*>(x));
    return hipGetLastError();
}

// Rotary embedding, half-split pairing (element i with i + d/2), angle = position * base^(-2i/d), at
// the ORIGINAL absolute position of the token (a bypassed token leaves a gap in the positions seen by
// a layer).  One workgroup per executed row: the d/2 (cos, sin) pairs of the row's position are
// evaluated once in fp64 into LDS, then every thread rotates 8 pairs of one q or k head with 16-byte
// accesses.  With a cache, rotated k and v are also appended at kv_old[seq] + (rank of the row inside
// its sequence), one head_dim-wide piece per kv head.
__global__ void __launch_bounds__(256)
rope_append_kernel(RopeArgs a) {
    __shared__ float cs[64], sn[64];              // head_dim <= 128
    const int i = blockIdx.x;
    if (i >= *a.count) return;
    const int t = a.idx[i];
    const int d = a.d, half = d >> 1;
    const int width = (a.nh + 2 * a.nkv) * d;
    half_t* row = reinterpret_cast<half_t*>(a.qkv) + static_cast<size_t>(i) * width;
    // cache layout [B][n_kv_heads][cap][d]: entry (b, head, slot) starts at ((b * nkv + head) * cap + slot) * d
    half_t* kdst = nullptr;                       // entry (b, head 0, slot); heads are head_step halves apart
    half_t* vdst = nullptr;
    const size_t head_step = static_cast<size_t>(a.cap) * d;
    if (a.k_cache) {
        const int b = a.row_seq[i];
        const int slot = a.kv_old[b] + (i - a.cu_exec[b]);
        if (slot < a.cap) {
            const size_t off = (static_cast<size_t>(b) * a.nkv * a.cap + slot) * d;
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
            *reinterpret_cast<half8_t*>(kdst + (hd - a.nh) * head_step + p0) = rlo;
            *reinterpret_cast<half8_t*>(kdst + (hd - a.nh) * head_step + p0 + half) = rhi;
        }
    }
    if (vdst) {
        const half8_t* vsrc = reinterpret_cast<const half8_t*>(row + static_cast<size_t>(a.nh + a.nkv) * d);
        const int cpr = d >> 3;                    // 16-byte chunks per head
        for (int e = threadIdx.x; e < a.nkv * cpr; e += blockDim.x)
            *reinterpret_cast<half8_t*>(vdst + (e / cpr) * head_step + (e % cpr) * 8) = vsrc[e];
    }
}

hipError_t launch_rope_append(const RopeArgs& a, hipStream_t stream) {
    if (a.max_rows == 0) return hipSuccess;
    hipLaunchKernelGGL(rope_append_kernel, dim3(a.max_rows), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace qtale
