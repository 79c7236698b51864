// Router score, threshold / top-k selection and order-preserving compaction (Eq. 2, Eq. 9, App. B.2).
//
// Score: z_t = fp32( sum_h fp64(x[t,h]) * fp64(w[h]) + fp64(b) ).  Products of a 16-bit activation and an
// fp32 weight are exact in fp64, so the only order-dependent error is the fp64 summation, far below
// the final fp32 rounding; the decision is then taken on the fp32 bit patterns, which makes the
// executed set reproducible.
// Decision (logit domain; sigmoid is strictly increasing so p_0 >= theta <=> z >= logit(theta)):
//   threshold mode: execute iff z >= z_thr;
//   ratio mode:     execute the k largest z, equal scores to the lower token index.
#include "qtale_dev.h"
#include "qtale_kernels.h"

namespace qtale {

template <bool BF16>
__global__ void __launch_bounds__(256)
router_score_kernel(const uint16_t* __restrict__ x, int T, int H, const float* __restrict__ w, float b,
                    float* __restrict__ z) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const U4* xr = reinterpret_cast<const U4*>(x + static_cast<size_t>(t) * H);
    const float4* wr = reinterpret_cast<const float4*>(w);
    double acc0 = 0.0, acc1 = 0.0;
    const int chunks = H >> 3;
    for (int c = lane; c < chunks; c += 64) {
        const U4 xv = xr[c];
        const float4 w0 = wr[2 * c], w1 = wr[2 * c + 1];
        const uint32_t xs[4] = {xv.x, xv.y, xv.z, xv.w};
        const float ws[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const double a0 = static_cast<double>(act_to_float<BF16>(static_cast<uint16_t>(xs[i] & 0xffffu)));
            const double a1 = static_cast<double>(act_to_float<BF16>(static_cast<uint16_t>(xs[i] >> 16)));
            acc0 = fma(a0, static_cast<double>(ws[2 * i]), acc0);
            acc1 = fma(a1, static_cast<double>(ws[2 * i + 1]), acc1);
        }
    }
    double acc = wave_sum(acc0 + acc1);
    if (lane == 0) z[t] = static_cast<float>(acc + static_cast<double>(b));
}

hipError_t launch_router_score(const void* x, int bf16, int T, int H, const float* w, float b, float* z,
                               hipStream_t stream) {
    if (T == 0) return hipSuccess;
    const dim3 grid((T + 3) / 4), block(256);
    if (bf16)
        hipLaunchKernelGGL(router_score_kernel<true>, grid, block, 0, stream,
                           reinterpret_cast<const uint16_t*>(x), T, H, w, b, z);
    else
        hipLaunchKernelGGL(router_score_kernel<false>, grid, block, 0, stream,
                           reinterpret_cast<const uint16_t*>(x), T, H, w, b, z);
    return hipGetLastError();
}

// Last kernel of a decode-sized layer inside a stack, fused with the next layer's router: one wave per token.  An
// executed token's row is h + sum of the down-proj's K parts (in part order), rounded to the stream's dtype and stored;
// a bypassed token's row is read.  Either way the wave then holds the row as stored and accumulates the next layer's
// score exactly as router_score_kernel does (same chunks per lane, same two fp64 accumulators, same wave sum).
template <bool BF16>
__global__ void __launch_bounds__(64)
scatter_score_kernel(const float* __restrict__ part, int n_parts, size_t part_stride, const float* __restrict__ h, int H,
                     const int32_t* __restrict__ inv, uint16_t* __restrict__ x, const float* __restrict__ w, float b,
                     float* __restrict__ z) {
    const int lane = threadIdx.x;
    const int t = blockIdx.x;
    const int row = inv[t];
    U4* xr = reinterpret_cast<U4*>(x + static_cast<size_t>(t) * H);
    const float4* wr = reinterpret_cast<const float4*>(w);
    const float4* hr = reinterpret_cast<const float4*>(h + static_cast<size_t>(row < 0 ? 0 : row) * H);
    const float4* pr = reinterpret_cast<const float4*>(part + static_cast<size_t>(row < 0 ? 0 : row) * H);
    const size_t pstep = part_stride / 4;
    double acc0 = 0.0, acc1 = 0.0;
    const int chunks = H >> 3;
    constexpr int U = 4;                                         // chunks whose loads are in flight together
    for (int c0 = lane; c0 < chunks; c0 += 64 * U) {
        U4 xv[U];
        float4 w0[U], w1[U];
        if (row >= 0) {
            float4 lo[U], hi[U], pl[U][kGemmPartMax], ph[U][kGemmPartMax];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = min(c0 + 64 * u, chunks - 1);
                lo[u] = hr[2 * c]; hi[u] = hr[2 * c + 1];
                w0[u] = wr[2 * c]; w1[u] = wr[2 * c + 1];
#pragma unroll
                for (int s = 0; s < kGemmPartMax; ++s) {
                    const size_t o = (s < n_parts ? s : 0) * pstep;
                    pl[u][s] = pr[o + 2 * c];
                    ph[u][s] = pr[o + 2 * c + 1];
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float4 sl = pl[u][0], sh = ph[u][0];
#pragma unroll
                for (int s = 1; s < kGemmPartMax; ++s)
                    if (s < n_parts) {
                        sl.x += pl[u][s].x; sl.y += pl[u][s].y; sl.z += pl[u][s].z; sl.w += pl[u][s].w;
                        sh.x += ph[u][s].x; sh.y += ph[u][s].y; sh.z += ph[u][s].z; sh.w += ph[u][s].w;
                    }
                const float4 l = lo[u], g = hi[u];
                const float v[8] = {l.x + sl.x, l.y + sl.y, l.z + sl.z, l.w + sl.w, g.x + sh.x, g.y + sh.y, g.z + sh.z, g.w + sh.w};
                xv[u].x = static_cast<uint32_t>(float_to_act<BF16>(v[0])) | (static_cast<uint32_t>(float_to_act<BF16>(v[1])) << 16);
                xv[u].y = static_cast<uint32_t>(float_to_act<BF16>(v[2])) | (static_cast<uint32_t>(float_to_act<BF16>(v[3])) << 16);
                xv[u].z = static_cast<uint32_t>(float_to_act<BF16>(v[4])) | (static_cast<uint32_t>(float_to_act<BF16>(v[5])) << 16);
                xv[u].w = static_cast<uint32_t>(float_to_act<BF16>(v[6])) | (static_cast<uint32_t>(float_to_act<BF16>(v[7])) << 16);
                if (c0 + 64 * u < chunks) xr[c0 + 64 * u] = xv[u];
            }
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = min(c0 + 64 * u, chunks - 1);
                xv[u] = xr[c];
                w0[u] = wr[2 * c]; w1[u] = wr[2 * c + 1];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (c0 + 64 * u >= chunks) break;
            const uint32_t xs[4] = {xv[u].x, xv[u].y, xv[u].z, xv[u].w};
            const float ws[8] = {w0[u].x, w0[u].y, w0[u].z, w0[u].w, w1[u].x, w1[u].y, w1[u].z, w1[u].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const double a0 = static_cast<double>(act_to_float<BF16>(static_cast<uint16_t>(xs[i] & 0xffffu)));
                const double a1 = static_cast<double>(act_to_float<BF16>(static_cast<uint16_t>(xs[i] >> 16)));
                acc0 = fma(a0, static_cast<double>(ws[2 * i]), acc0);
                acc1 = fma(a1, static_cast<double>(ws[2 * i + 1]), acc1);
            }
        }
    }
    const double acc = wave_sum(acc0 + acc1);
    if (lane == 0) z[t] = static_cast<float>(acc + static_cast<double>(b));
}

hipError_t launch_reduce_scatter_score(const float* part, int n_parts, int part_rows, const float* h, int H, const int32_t* inv,
                                       int T, void* x, int bf16, const float* w_next, float b_next, float* z_next,
                                       hipStream_t stream) {
    if (T == 0) return hipSuccess;
    const size_t stride = static_cast<size_t>(part_rows) * H;
    if (bf16)
        hipLaunchKernelGGL(scatter_score_kernel<true>, dim3(T), dim3(64), 0, stream, part, n_parts, stride, h, H, inv,
                           reinterpret_cast<uint16_t*>(x), w_next, b_next, z_next);
    else
        hipLaunchKernelGGL(scatter_score_kernel<false>, dim3(T), dim3(64), 0, stream, part, n_parts, stride, h, H, inv,
                           reinterpret_cast<uint16_t*>(x), w_next, b_next, z_next);
    return hipGetLastError();
}

// Two-output MLP router (Sec. 2.2: "lightweight MLP" with two outputs; Eq. 9 takes their softmax).  This
// library's reading: one hidden ReLU layer,  u = relu(W1 x + b1),  (l_e, l_b) = W2 u + b2,  score
// z = l_e - l_b (the two-class softmax gives p_0 = sigmoid(z)).  All sums in fp64, one rounding to fp32, so
// the executed set is reproducible exactly as for the linear router.
//
// The first layer is a [T x H] x [H x R] product in fp64 on the vector ALUs.  A workgroup owns 16 tokens (four
// per wave) and walks H in chunks of 512 columns: the W1 chunk of 4 hidden units is staged in LDS once per
// workgroup (two buffers, the next chunk's global loads are issued before the current one is consumed, one
// barrier per chunk), a lane holds 8 consecutive columns of its four tokens, and every staged weight is
// converted to fp64 once and used for four tokens (16 accumulators of two registers each per lane, two
// workgroups per CU; 8 units per pass would spill).  The walk repeats per group of 4 units (x then comes
// from L2).
constexpr int kMlpRC = 4;         // hidden units per pass
constexpr int kMlpKC = 512;       // columns per staged chunk
constexpr int kMlpTW = 4;         // tokens per wave
constexpr int kMlpWL = (kMlpRC * kMlpKC / 4) / 256;   // float4 loads per thread per chunk

template <bool BF16>
__global__ void __launch_bounds__(256, 2)
router_mlp_kernel(const uint16_t* __restrict__ x, int T, int H, const float* __restrict__ W1,
                  const float* __restrict__ b1, const float* __restrict__ W2, const float* __restrict__ b2, int R,
                  float* __restrict__ z) {
    __shared__ __attribute__((aligned(16))) float Ws[2][kMlpRC][kMlpKC];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = blockIdx.x * (4 * kMlpTW) + wave * kMlpTW;
    const uint16_t* xrow[kMlpTW];
#pragma unroll
    for (int i = 0; i < kMlpTW; ++i) xrow[i] = x + static_cast<size_t>(min(t0 + i, T - 1)) * H;

    double le[kMlpTW], lb[kMlpTW];
#pragma unroll
    for (int i = 0; i < kMlpTW; ++i) { le[i] = 0.0; lb[i] = 0.0; }

    float4 wreg[kMlpWL];
    u32x4_t xreg[kMlpTW];
    auto fetch = [&](int rc, int kb) {                         // global -> registers for chunk (rc, kb)
#pragma unroll
        for (int it = 0; it < kMlpWL; ++it) {
            const int c = it * 256 + tid;
            const int row = c / (kMlpKC / 4), col = (c % (kMlpKC / 4)) * 4;
            wreg[it] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (rc + row < R && kb + col < H)
                wreg[it] = *reinterpret_cast<const float4*>(W1 + static_cast<size_t>(rc + row) * H + kb + col);
        }
        const int k = kb + lane * 8;
#pragma unroll
        for (int i = 0; i < kMlpTW; ++i) {
            xreg[i] = u32x4_t{0u, 0u, 0u, 0u};
            if (k < H) xreg[i] = *reinterpret_cast<const u32x4_t*>(xrow[i] + k);
        }
    };

    const int n_kb = (H + kMlpKC - 1) / kMlpKC;
    const int n_rc = (R + kMlpRC - 1) / kMlpRC;
    const int n_chunks = n_rc * n_kb;                          // walked as one sequence: rc-major, kb-minor
    fetch(0, 0);
    int buf = 0;
    double acc[kMlpTW][kMlpRC];
    for (int ch = 0; ch < n_chunks; ++ch) {
        const int rc = (ch / n_kb) * kMlpRC, kbi = ch % n_kb;
        if (kbi == 0) {
#pragma unroll
            for (int i = 0; i < kMlpTW; ++i)
#pragma unroll
                for (int r = 0; r < kMlpRC; ++r) acc[i][r] = 0.0;
        }
        // park this chunk's weights, expand this chunk's activations
#pragma unroll
        for (int it = 0; it < kMlpWL; ++it) {
            const int c = it * 256 + tid;
            *reinterpret_cast<float4*>(&Ws[buf][c / (kMlpKC / 4)][(c % (kMlpKC / 4)) * 4]) = wreg[it];
        }
        double xd[kMlpTW][8];
#pragma unroll
        for (int i = 0; i < kMlpTW; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                xd[i][2 * j] = static_cast<double>(act_to_float<BF16>(static_cast<uint16_t>(xreg[i][j] & 0xffffu)));
                xd[i][2 * j + 1] = static_cast<double>(act_to_float<BF16>(static_cast<uint16_t>(xreg[i][j] >> 16)));
            }
        __syncthreads();          // chunk staged; the other buffer (read in the previous iteration) is free again
        if (ch + 1 < n_chunks) fetch(((ch + 1) / n_kb) * kMlpRC, ((ch + 1) % n_kb) * kMlpKC);
#pragma unroll
        for (int r = 0; r < kMlpRC; ++r) {
            const float4 w0 = *reinterpret_cast<const float4*>(&Ws[buf][r][lane * 8]);
            const float4 w1 = *reinterpret_cast<const float4*>(&Ws[buf][r][lane * 8 + 4]);
            const double wd[8] = {static_cast<double>(w0.x), static_cast<double>(w0.y), static_cast<double>(w0.z),
                                  static_cast<double>(w0.w), static_cast<double>(w1.x), static_cast<double>(w1.y),
                                  static_cast<double>(w1.z), static_cast<double>(w1.w)};
#pragma unroll
            for (int i = 0; i < kMlpTW; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i][r] = fma(xd[i][j], wd[j], acc[i][r]);
        }
        buf ^= 1;
        if (kbi == n_kb - 1) {
            // hidden units of this pass: full sums, bias, ReLU, then their share of the two logits (in unit order)
#pragma unroll
            for (int r = 0; r < kMlpRC; ++r) {
                const bool live = rc + r < R;
                const double bias = live ? static_cast<double>(b1[rc + r]) : 0.0;
                const double we = live ? static_cast<double>(W2[rc + r]) : 0.0;
                const double wb = live ? static_cast<double>(W2[R + rc + r]) : 0.0;
#pragma unroll
                for (int i = 0; i < kMlpTW; ++i) {
                    const double u = fmax(wave_sum(acc[i][r]) + bias, 0.0);
                    le[i] = fma(we, u, le[i]);
                    lb[i] = fma(wb, u, lb[i]);
                }
            }
        }
    }
    if (lane == 0) {
        const double be = static_cast<double>(b2[0]), bb = static_cast<double>(b2[1]);
#pragma unroll
        for (int i = 0; i < kMlpTW; ++i)
            if (t0 + i < T) z[t0 + i] = static_cast<float>((le[i] + be) - (lb[i] + bb));
    }
}

// Few tokens (decode steps): one workgroup per token, the 256 threads split H (8 columns each per 2048-column
// sweep) and read W1 straight from L2, 16 hidden units per pass with 4 units' loads in flight; the per-thread
// partial sums meet in a wave reduction plus a four-entry LDS exchange.
template <bool BF16>
__global__ void __launch_bounds__(256)
router_mlp_small_kernel(const uint16_t* __restrict__ x, int T, int H, const float* __restrict__ W1,
                        const float* __restrict__ b1, const float* __restrict__ W2, const float* __restrict__ b2, int R,
                        float* __restrict__ z) {
    constexpr int RG = 16;
    __shared__ double part[4][RG];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t = blockIdx.x;
    const uint16_t* xr = x + static_cast<size_t>(t) * H;
    double le = 0.0, lb = 0.0;
    for (int rg = 0; rg < R; rg += RG) {
        double acc[RG];
#pragma unroll
        for (int r = 0; r < RG; ++r) acc[r] = 0.0;
        for (int k = tid * 8; k < H; k += 2048) {
            const u32x4_t xv = *reinterpret_cast<const u32x4_t*>(xr + k);
            double xd[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                xd[2 * j] = static_cast<double>(act_to_float<BF16>(static_cast<uint16_t>(xv[j] & 0xffffu)));
                xd[2 * j + 1] = static_cast<double>(act_to_float<BF16>(static_cast<uint16_t>(xv[j] >> 16)));
            }
#pragma unroll
            for (int r4 = 0; r4 < RG; r4 += 4) {
                float4 w[4][2];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int r = min(rg + r4 + u, R - 1);     // rows past R repeat the last one; their sums are dropped
                    const float4* wp = reinterpret_cast<const float4*>(W1 + static_cast<size_t>(r) * H + k);
                    w[u][0] = wp[0];
                    w[u][1] = wp[1];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float wf[8] = {w[u][0].x, w[u][0].y, w[u][0].z, w[u][0].w, w[u][1].x, w[u][1].y, w[u][1].z, w[u][1].w};
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[r4 + u] = fma(xd[j], static_cast<double>(wf[j]), acc[r4 + u]);
                }
            }
        }
        __syncthreads();                                       // `part` of the previous group has been read
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            const double v = wave_sum(acc[r]);
            if (lane == 0) part[wave][r] = v;
        }
        __syncthreads();
        if (tid == 0) {
            for (int r = 0; r < RG && rg + r < R; ++r) {
                const double sum = (part[0][r] + part[1][r]) + (part[2][r] + part[3][r]);
                const double u = fmax(sum + static_cast<double>(b1[rg + r]), 0.0);
                le = fma(static_cast<double>(W2[rg + r]), u, le);
                lb = fma(static_cast<double>(W2[R + rg + r]), u, lb);
            }
        }
    }
    if (tid == 0) z[t] = static_cast<float>((le + static_cast<double>(b2[0])) - (lb + static_cast<double>(b2[1])));
}

hipError_t launch_router_mlp(const void* x, int bf16, int T, int H, const float* W1, const float* b1, const float* W2,
                             const float* b2, int R, float* z, hipStream_t stream) {
    if (T == 0) return hipSuccess;
    const uint16_t* xp = reinterpret_cast<const uint16_t*>(x);
    if (T <= 512) {                                            // too few tokens to fill the chip 16 per workgroup
        if (bf16)
            hipLaunchKernelGGL(router_mlp_small_kernel<true>, dim3(T), dim3(256), 0, stream, xp, T, H, W1, b1, W2, b2, R, z);
        else
            hipLaunchKernelGGL(router_mlp_small_kernel<false>, dim3(T), dim3(256), 0, stream, xp, T, H, W1, b1, W2, b2, R, z);
        return hipGetLastError();
    }
    const dim3 grid((T + 4 * kMlpTW - 1) / (4 * kMlpTW)), block(256);
    if (bf16)
        hipLaunchKernelGGL(router_mlp_kernel<true>, grid, block, 0, stream, xp, T, H, W1, b1, W2, b2, R, z);
    else
        hipLaunchKernelGGL(router_mlp_kernel<false>, grid, block, 0, stream, xp, T, H, W1, b1, W2, b2, R, z);
    return hipGetLastError();
}

// fp32 -> uint32 key whose unsigned order is the float order (-0 is first folded onto +0).  A NaN score gets the
// smallest key: it ranks below every number, also below -inf, so it never meets a threshold (as in
// threshold_bins_kernel) and is taken by the ratio rule only after every other token.
__device__ __forceinline__ uint32_t order_key(float f) {
    f += 0.0f;
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <int kSelThreads>
__device__ __forceinline__ uint32_t block_scan_inclusive(uint32_t v, uint32_t* wsum, uint32_t& total) {
    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(v, o, 64);
        if (lane >= o) v += t;
    }
    if (lane == 63) wsum[wid] = v;
    __syncthreads();
    if (wid == 0) {
        uint32_t w = lane < (kSelThreads / 64) ? wsum[lane] : 0u;
#pragma unroll
        for (int o = 1; o < kSelThreads / 64; o <<= 1) {
            const uint32_t t = __shfl_up(w, o, 64);
            if (lane >= o) w += t;
        }
        if (lane < kSelThreads / 64) wsum[lane] = w;
    }
    __syncthreads();
    if (wid > 0) v += wsum[wid - 1];
    total = wsum[kSelThreads / 64 - 1];
    __syncthreads();
    return v;
}

// One workgroup selects and compacts: four 8-bit radix passes find the k-th largest key, one ordered
// pass writes ascending indices, the tail derives per-sequence counts and advances the cache lengths.
// Everything that is touched more than once lives in LDS (keys of up to 16384 tokens, up to 2048 sequence
// offsets, the per-thread prefix counts of the current chunk): a single workgroup has nothing to hide the
// latency of dependent global loads with, and binary searches over global arrays used to dominate its time.
constexpr int kSelKeyCache = 16384;
constexpr int kSelOffCache = 2048;
constexpr int kSelPer = 8;                       // consecutive tokens per thread in the ordered pass

template <int kSelThreads>
__global__ void __launch_bounds__(kSelThreads)
select_compact_kernel(SelectArgs a) {
    extern __shared__ uint32_t skeys[];           // T keys when T <= kSelKeyCache (sized at launch)
    __shared__ int32_t soffs[kSelOffCache];
    __shared__ int32_t scu[kSelOffCache];        // executed tokens before each sequence boundary
    __shared__ uint32_t pre[kSelThreads];        // executed tokens before the thread's first token (whole call)
    __shared__ uint32_t emask[kSelThreads];      // which of the thread's tokens execute
    __shared__ uint32_t hist[2][256];            // radix pass p counts into hist[p & 1] while the other one is cleared
    __shared__ uint32_t wsum[kSelThreads / 64];
    __shared__ uint32_t s_prefix, s_krem;
    const int tid = threadIdx.x;
    const int T = a.T;
    const bool keys_cached = T <= kSelKeyCache;
    const bool offs_cached = a.B >= 0 && a.B + 1 <= kSelOffCache;
    if (keys_cached)
        for (int t = tid; t < T; t += kSelThreads) skeys[t] = order_key(a.z[t]);
    if (offs_cached)
        for (int b = tid; b <= a.B; b += kSelThreads) soffs[b] = a.seq_offsets[b];
    for (int i = tid; i < 256; i += kSelThreads) hist[0][i] = 0u;
    __syncthreads();
    auto key_of = [&](int t) { return keys_cached ? skeys[t] : order_key(a.z[t]); };
    auto off_of = [&](int b) { return offs_cached ? soffs[b] : a.seq_offsets[b]; };
    auto put_cu = [&](int b, int v) {
        if (offs_cached) scu[b] = v;
        if (a.cu_exec) a.cu_exec[b] = v;
    };

    uint32_t kth, need_eq;
    if (a.mode == 0) {
        if (a.k <= 0) {
            kth = 0xffffffffu;
            need_eq = 0u;
        } else {
            uint32_t prefix = 0u, krem = static_cast<uint32_t>(a.k);
            for (int pass = 0; pass < 4; ++pass) {
                const int shift = 24 - 8 * pass;
                uint32_t* h = hist[pass & 1];
                for (int i = tid; i < 256; i += kSelThreads) hist[(pass + 1) & 1][i] = 0u;
                for (int t = tid; t < T; t += kSelThreads) {
                    const uint32_t key = key_of(t);
                    if (pass == 0 || (key >> (shift + 8)) == prefix) atomicAdd(&h[(key >> shift) & 255u], 1u);
                }
                __syncthreads();
                if (tid < 64) {
                    const uint32_t h0 = h[4 * tid], h1 = h[4 * tid + 1], h2 = h[4 * tid + 2], h3 = h[4 * tid + 3];
                    const uint32_t s = h0 + h1 + h2 + h3;
                    uint32_t suf = s;                        // inclusive sum over lanes >= tid
#pragma unroll
                    for (int o = 1; o < 64; o <<= 1) {
                        const uint32_t t = __shfl_down(suf, o, 64);
                        if (tid + o < 64) suf += t;
                    }
                    const uint32_t above = suf - s;          // keys with a larger digit than this lane's bins
                    if (above < krem && krem <= above + s) {
                        uint32_t cum = above;
                        int d;
                        if (cum + h3 >= krem) d = 3;
                        else { cum += h3; if (cum + h2 >= krem) d = 2;
                        else { cum += h2; if (cum + h1 >= krem) d = 1;
                        else { cum += h1; d = 0; } } }
                        s_prefix = (prefix << 8) | static_cast<uint32_t>(4 * tid + d);
                        s_krem = krem - cum;
                    }
                }
                __syncthreads();                             // s_prefix / s_krem are rewritten only after the next
                prefix = s_prefix;                           // pass's first barrier
                krem = s_krem;
            }
            kth = prefix;
            need_eq = krem;
        }
    } else {
        kth = order_key(a.z_thr);
        need_eq = 0x7fffffffu;
    }

    // Ordered compaction.  A thread owns `per` (up to 8) consecutive tokens, so one block scan of the per-thread
    // counts (executed-by-score in the low half, ties in the high half) orders a chunk of threads x per tokens.  The
    // thread's prefix count and execute mask stay in LDS for the boundary pass below: the executed tokens
    // before a sequence boundary are the prefix of the thread that owns the boundary token plus the set bits
    // below it, so no search over the index list is needed.
    const int per = min(kSelPer, (T + kSelThreads - 1) / kSelThreads);
    uint32_t base_gt = 0u, base_eq = 0u;
    for (int c0 = 0; c0 < T; c0 += kSelThreads * per) {
        const int t0 = c0 + tid * per;
        uint32_t gtm = 0u, eqm = 0u;
#pragma unroll
        for (int j = 0; j < kSelPer; ++j) {
            if (j < per && t0 + j < T) {
                const uint32_t key = key_of(t0 + j);
                gtm |= (key > kth ? 1u : 0u) << j;
                eqm |= (key == kth ? 1u : 0u) << j;
            }
        }
        const uint32_t packed = static_cast<uint32_t>(__popc(gtm)) | (static_cast<uint32_t>(__popc(eqm)) << 16);
        uint32_t total;
        const uint32_t excl = block_scan_inclusive<kSelThreads>(packed, wsum, total) - packed;
        uint32_t gt_before = base_gt + (excl & 0xffffu);
        uint32_t eq_before = base_eq + (excl >> 16);
        pre[tid] = gt_before + (eq_before < need_eq ? eq_before : need_eq);
        int seq = -1;                                       // sequence of the previous executed token of this thread
        uint32_t em = 0u;
#pragma unroll
        for (int j = 0; j < kSelPer; ++j) {
            const uint32_t gt = (gtm >> j) & 1u, eq = (eqm >> j) & 1u;
            if (gt || (eq && eq_before < need_eq)) {
                const uint32_t pos = gt_before + (eq_before < need_eq ? eq_before : need_eq);
                const int t = t0 + j;
                em |= 1u << j;
                a.idx[pos] = t;
                if (a.idx_copy) a.idx_copy[pos] = t;
                if (a.row_seq) {
                    if (seq < 0 || off_of(seq + 1) <= t) {  // left the previous token's sequence: search again
                        int lo = 0, hi = a.B;               // last b with seq_offsets[b] <= t
                        while (lo + 1 < hi) {
                            const int mid = (lo + hi) >> 1;
                            if (off_of(mid) <= t) lo = mid; else hi = mid;
                        }
                        seq = lo;
                    }
                    a.row_seq[pos] = seq;
                }
            }
            gt_before += gt;
            eq_before += eq;
        }
        emask[tid] = em;
        __syncthreads();
        // sequence boundaries that fall into this chunk
        {
            const int c1 = min(c0 + kSelThreads * per, T);
            for (int b = tid; b <= a.B; b += kSelThreads) {
                const int o = off_of(b);
                if (o >= c0 && o < c1) {
                    const int owner = (o - c0) / per, below = (o - c0) % per;
                    put_cu(b, static_cast<int>(pre[owner] + __popc(emask[owner] & ((1u << below) - 1u))));
                }
            }
        }
        base_gt += total & 0xffffu;
        base_eq += total >> 16;
        __syncthreads();                                    // pre / emask are rewritten by the next chunk
    }
    const int count = static_cast<int>(base_gt + (base_eq < need_eq ? base_eq : need_eq));
    if (tid == 0) {
        *a.count = count;
        if (a.count_copy) *a.count_copy = count;
    }
    for (int b = tid; b <= a.B; b += kSelThreads)
        if (off_of(b) >= T) put_cu(b, count);               // boundaries at the end of the call
    __syncthreads();
    if (a.kv_len) {                                         // cu_exec is given whenever the sequence table is too long for LDS
        for (int b = tid; b < a.B; b += kSelThreads) {
            const int cb = offs_cached ? scu[b] : a.cu_exec[b];
            const int cn = offs_cached ? scu[b + 1] : a.cu_exec[b + 1];
            const int old = a.kv_len[b];
            a.kv_old[b] = old;
            // entries that do not fit are dropped by the append; the length never passes the capacity
            a.kv_len[b] = a.kv_cap > 0 ? min(old + (cn - cb), max(old, a.kv_cap)) : old + (cn - cb);
        }
    }
}

hipError_t launch_select(const SelectArgs& a, hipStream_t stream) {
    const size_t key_bytes = a.T <= kSelKeyCache ? static_cast<size_t>(a.T > 0 ? a.T : 0) * 4 : 0;
    if (a.T <= 2048)       // few tokens (decode steps): four waves, cheaper barriers
        hipLaunchKernelGGL(select_compact_kernel<256>, dim3(1), dim3(256), key_bytes, stream, a);
    else
        hipLaunchKernelGGL(select_compact_kernel<1024>, dim3(1), dim3(1024), key_bytes, stream, a);
    return hipGetLastError();
}

// ---- decode-sized calls: decision, compaction and the first normalisation in ONE launch -------------------------
// With a few dozen tokens (a decode step: one token per sequence) selection and gather + RMSNorm as two launches are
// pure launch and latency cost.  Here workgroup i produces compact row i on its own:
//   1. every workgroup reads the T scores the router kernel wrote (Eq. 2) and turns them into order keys in LDS;
//   2. every workgroup takes the decision (Eq. 9 / the k largest, ties to the lower index) on those keys: rank by
//      counting, exclusive prefix of the executed flags by counting;
//   3. workgroup i normalises the row of the i-th executed token (App. B.2 gather + RMSNorm); workgroup 0 also writes the
//      call-wide results (ascending indices, count, per-sequence offsets, row -> sequence map, cache lengths).
// The redundant decision costs T LDS reads per thread, which bounds T (kFusedMaxT).
constexpr int kFusedMaxT = 256;

struct FusedArgs {
    const uint16_t* x; int H; const float* z; const uint16_t* gain; float eps; uint16_t* out;
    SelectArgs s;
};

template <bool BF16>
__global__ void __launch_bounds__(256)
select_norm_kernel(FusedArgs a) {
    __shared__ __align__(16) uint32_t skey[kFusedMaxT];
    __shared__ uint32_t spre[kFusedMaxT + 1];
    __shared__ unsigned long long smask[4];
    __shared__ int srow;
    __shared__ float red[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int T = a.s.T, H = a.H;
    const int chunks = H >> 3;
    // 1. order keys of the scores the router kernel left in z (0 = below every real key for the padding)
    skey[tid] = tid < T ? order_key(a.z[tid]) : 0u;
    __syncthreads();
    // 2. decision: threshold mode compares with the threshold's key, ratio mode ranks
    const uint32_t key = skey[tid];
    bool exec = false;
    if (a.s.mode == 0) {
        uint32_t rank = 0u;
        const int T4 = (T + 3) >> 2;
        const uint4* k4 = reinterpret_cast<const uint4*>(skey);
#pragma unroll 4
        for (int q = 0; q < T4; ++q) {                              // same address in every lane: LDS broadcast reads
            const uint4 kk = k4[q];
            const int u = q << 2;
            rank += (kk.x > key || (kk.x == key && u < tid)) ? 1u : 0u;
            rank += (kk.y > key || (kk.y == key && u + 1 < tid)) ? 1u : 0u;
            rank += (kk.z > key || (kk.z == key && u + 2 < tid)) ? 1u : 0u;
            rank += (kk.w > key || (kk.w == key && u + 3 < tid)) ? 1u : 0u;
        }
        exec = tid < T && static_cast<int>(rank) < a.s.k;
    } else {
        exec = tid < T && key >= order_key(a.s.z_thr);
    }
    const unsigned long long mask = __ballot(exec);
    if (lane == 0) smask[wave] = mask;
    __syncthreads();
    int before = __popcll(mask & ((1ull << lane) - 1ull));         // executed tokens before token tid
    for (int v = 0; v < wave; ++v) before += __popcll(smask[v]);
    const int count = __popcll(smask[0]) + __popcll(smask[1]) + __popcll(smask[2]) + __popcll(smask[3]);
    if (tid < T) spre[tid] = static_cast<uint32_t>(before);
    if (tid == 0) spre[T] = static_cast<uint32_t>(count);
    if (exec && before == static_cast<int>(blockIdx.x)) srow = tid; // the row this workgroup normalises
    __syncthreads();
    if (blockIdx.x == 0) {
        if (tid == 0) {
            *a.s.count = count;
            if (a.s.count_copy) *a.s.count_copy = count;
        }
        if (a.s.inv && tid < T) a.s.inv[tid] = exec ? before : -1;
        if (exec) {
            const int pos = before;
            a.s.idx[pos] = tid;
            if (a.s.idx_copy) a.s.idx_copy[pos] = tid;
            if (a.s.row_seq) {
                int lo = 0, hi = a.s.B;                             // last b with seq_offsets[b] <= t
                while (lo + 1 < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (a.s.seq_offsets[mid] <= tid) lo = mid; else hi = mid;
                }
                a.s.row_seq[pos] = lo;
            }
        }
        for (int b = tid; b <= a.s.B; b += 256) {
            const int o = a.s.seq_offsets[b];
            if (a.s.cu_exec) a.s.cu_exec[b] = o >= T ? count : static_cast<int>(spre[o]);
        }
        if (a.s.kv_len) {
            for (int b = tid; b < a.s.B; b += 256) {
                const int o0 = a.s.seq_offsets[b], o1 = a.s.seq_offsets[b + 1];
                const int n = (o1 >= T ? count : static_cast<int>(spre[o1])) - (o0 >= T ? count : static_cast<int>(spre[o0]));
                const int old = a.s.kv_len[b];
                a.s.kv_old[b] = old;
                a.s.kv_len[b] = a.s.kv_cap > 0 ? min(old + n, max(old, a.s.kv_cap)) : old + n;
            }
        }
    }
    // 3. this workgroup's compact row
    const int i = blockIdx.x;
    if (i >= count) return;
    const int t = srow;
    const u32x4_t* xr = reinterpret_cast<const u32x4_t*>(a.x + static_cast<size_t>(t) * H);
    const u32x4_t* gr = reinterpret_cast<const u32x4_t*>(a.gain);
    u32x4_t* orow = reinterpret_cast<u32x4_t*>(a.out + static_cast<size_t>(i) * H);
    constexpr int KEEP = 4;
    u32x4_t keep[KEEP];
    float ss = 0.0f;
    auto sumsq = [&](const u32x4_t& v) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float p = act_to_float<BF16>(static_cast<uint16_t>(v[j] & 0xffffu));
            const float q = act_to_float<BF16>(static_cast<uint16_t>(v[j] >> 16));
            ss = fmaf(p, p, ss);
            ss = fmaf(q, q, ss);
        }
    };
#pragma unroll
    for (int u = 0; u < KEEP; ++u) {
        const int c = tid + u * 256;
        keep[u] = c < chunks ? xr[c] : u32x4_t{0u, 0u, 0u, 0u};
        sumsq(keep[u]);
    }
    for (int c = tid + KEEP * 256; c < chunks; c += 256) sumsq(xr[c]);
    ss = wave_sum(ss);
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    ss = red[0] + red[1] + red[2] + red[3];
    const float inv = 1.0f / sqrtf(ss / static_cast<float>(H) + a.eps);
    auto emit = [&](int c, const u32x4_t& v) {
        const u32x4_t g = gr[c];
        u32x4_t o;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float p = act_to_float<BF16>(static_cast<uint16_t>(v[j] & 0xffffu)) * inv *
                            act_to_float<BF16>(static_cast<uint16_t>(g[j] & 0xffffu));
            const float q = act_to_float<BF16>(static_cast<uint16_t>(v[j] >> 16)) * inv *
                            act_to_float<BF16>(static_cast<uint16_t>(g[j] >> 16));
            o[j] = static_cast<uint32_t>(float_to_half_bits(p)) | (static_cast<uint32_t>(float_to_half_bits(q)) << 16);
        }
        orow[c] = o;
    };
#pragma unroll
    for (int u = 0; u < KEEP; ++u) {
        const int c = tid + u * 256;
        if (c < chunks) emit(c, keep[u]);
    }
    for (int c = tid + KEEP * 256; c < chunks; c += 256) emit(c, xr[c]);
}

bool fused_select_norm_fits(int T, int max_rows) { return max_rows > 0 && T <= kFusedMaxT; }

hipError_t launch_select_norm(const void* x, int bf16, int H, const float* z, const void* gain, float eps, void* out_f16,
                              const SelectArgs& s, int max_rows, hipStream_t stream) {
    FusedArgs a{};
    a.x = reinterpret_cast<const uint16_t*>(x); a.H = H; a.z = z;
    a.gain = reinterpret_cast<const uint16_t*>(gain); a.eps = eps;
    a.out = reinterpret_cast<uint16_t*>(out_f16); a.s = s;
    if (bf16) hipLaunchKernelGGL(select_norm_kernel<true>, dim3(max_rows), dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(select_norm_kernel<false>, dim3(max_rows), dim3(256), 0, stream, a);
    return hipGetLastError();
}

// Threshold calibration (Sec. 3.4): for fixed scores, how many (layer, token) pairs would execute at each of
// the grid thresholds.  zthr[j] ascends with j; a score falls into bin b = number of thresholds it reaches,
// so the count at threshold j is the sum of bins j+1 .. NTHR.  Integer atomics only: deterministic.
__global__ void __launch_bounds__(256)
threshold_bins_kernel(const float* __restrict__ scores, long n, const float* __restrict__ zthr,
                      unsigned long long* __restrict__ bins) {
    __shared__ unsigned int local[kThetaGrid + 1];
    __shared__ float zt[kThetaGrid];
    for (int i = threadIdx.x; i <= kThetaGrid; i += blockDim.x) local[i] = 0u;
    for (int i = threadIdx.x; i < kThetaGrid; i += blockDim.x) zt[i] = zthr[i];
    __syncthreads();
    const long stride = static_cast<long>(gridDim.x) * blockDim.x;
    for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride) {
        const float z = scores[i];
        int lo = 0, hi = kThetaGrid;                 // first j with !(z >= zthr[j]); NaN reaches none
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (z >= zt[mid]) lo = mid + 1; else hi = mid;
        }
        atomicAdd(&local[lo], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i <= kThetaGrid; i += blockDim.x)
        if (local[i]) atomicAdd(&bins[i], static_cast<unsigned long long>(local[i]));
}

hipError_t launch_threshold_bins(const float* scores, long n, const float* zthr_dev, unsigned long long* bins,
                                 hipStream_t stream) {
    hipError_t e = hipMemsetAsync(bins, 0, (kThetaGrid + 1) * sizeof(unsigned long long), stream);
    if (e != hipSuccess) return e;
    if (n == 0) return hipSuccess;
    long blocks = (n + 256L * 8 - 1) / (256L * 8);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(threshold_bins_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream, scores, n,
                       zthr_dev, bins);
    return hipGetLastError();
}

}  // namespace qtale
