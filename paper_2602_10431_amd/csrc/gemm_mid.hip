// W4A16 / W3A16 / W2A16 GEMM for the row counts between the decode kernel and the large-tile prefill kernel:
// a few hundred to about a thousand executed rows (a single prompt at a moderate execution ratio, Sec. 4.1
// weights on the rows gathered per App. B.2) times a narrow output (o-proj, down-proj: hidden-size columns).
//
// There the 128 x 256 tiles of the prefill kernel number fewer than the CUs, every CU holds at most one
// workgroup, and that workgroup's k-loop is a latency chain: its weight loads are issued one k-tile ahead and
// a k-tile of matrix-core work (well under 0.5 us) is shorter than the trip to L2/HBM, so each k-tile costs
// one memory latency (measured: 58 us for a 4096 x 4096 linear at any row count from 257 to 1024).  This
// kernel is built for that regime:
//   * workgroup tile 64 (M) x 128 (N): four waves, each 64 rows x one 32-column weight fragment; four times
//     as many workgroups as the large tiles, and few registers per wave (32 accumulators), so
//   * weights and activations are requested D = 4 k-tiles ahead (register rings, the loop is unrolled by D
//     so that ring slots are compile-time), which covers the memory latency with one workgroup per CU, and
//     up to four workgroups fit on a CU when there are that many;
//   * the rest is the prefill kernel's scheme: weights HBM/L2 -> VGPR -> dequantize -> MFMA, the A tile
//     through three LDS buffers with one barrier per k-tile, epilogues through `store_tile`.
// Workgroup ids are dealt round-robin to the 8 XCDs; the 64-row tiles of one 128-column panel get ids 8
// apart, so a weight panel is streamed into one L2 only.
#include "gemm_common.h"

namespace qtale {

template <int BITS, int FN, int D, int GPT, int EPI, bool RAGGED>
__global__ void __launch_bounds__(256, FN == 1 ? 3 : 2)
gemm_mid_kernel(GemmDev p) {
    using WB = WBits<BITS>;
    static_assert(EPI != EPI_SWIGLU_F16 || FN == 2, "a wave owns the gate and the up fragment of its output columns");
    constexpr int NT = 256;
    constexpr int FM = 2;
    constexpr int BM = FM * 32;
    constexpr int A_LOADS = (BM * 8) / NT;                      // 16-byte chunks per thread per k-tile
    constexpr int NBUF = 3;
    constexpr int kABytes = NBUF * BM * kLdsStride * 2;
    constexpr int kSlabFloats = 32 * ((EPI == EPI_SWIGLU_F16 ? FN / 2 : FN) * 32 + 8);
    constexpr int kCBytes = 4 * kSlabFloats * 4;
    __shared__ __attribute__((aligned(16))) char smem[kABytes > kCBytes ? kABytes : kCBytes];
    half_t (*As)[BM * kLdsStride] = reinterpret_cast<half_t (*)[BM * kLdsStride]>(smem);

    const int within = blockIdx.x % (8 * p.tiles_m);
    const int tile_n = (blockIdx.x / (8 * p.tiles_m)) * 8 + (within & 7);
    const int m0 = (within >> 3) * BM;
    if (tile_n >= p.tiles_n) return;
    const int M = p.count ? min(*p.count, p.M_max) : p.M_max;
    if (m0 >= M) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31;
    const int lhi = lane >> 5;
    const uint32_t magic = dequant_magic();

    const char* bbase[FN];
    const uint32_t* sbase[FN];
    int npad[FN];
#pragma unroll
    for (int fn = 0; fn < FN; ++fn) {
        int vf = (tile_n * 4 + wave) * FN + fn;
        if (vf >= p.vf_total) vf = p.vf_total - 1;             // edge tile: recompute the last fragment, never stored
        int mat, f;
        map_fragment<EPI>(p, vf, mat, f);
        bbase[fn] = reinterpret_cast<const char*>(p.codes[mat]) + static_cast<size_t>(f) * p.KT * (64 * WB::kLaneBytes);
        sbase[fn] = p.sz[mat] + f * 32;
        npad[fn] = p.npad[mat];
    }

    float16_t acc[FM][FN];
#pragma unroll
    for (int fm = 0; fm < FM; ++fm)
#pragma unroll
        for (int fn = 0; fn < FN; ++fn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[fm][fn][r] = 0.0f;

    // A tile: global -> registers (ring of D tiles) -> LDS.  Rows are clamped to M-1; with K not a multiple
    // of 64 (RAGGED) chunks of the last tile that start at or beyond K read the row's last valid chunk, whose
    // weights dequantize to exactly 0 (the prepacked layout pads with the zero-point).
    uint32_t a_off[A_LOADS];
    int a_dst[A_LOADS];
#pragma unroll
    for (int it = 0; it < A_LOADS; ++it) {
        const int c = it * NT + tid;
        const int row = c >> 3, col8 = c & 7;
        a_off[it] = static_cast<uint32_t>(min(m0 + row, M - 1)) * static_cast<uint32_t>(p.K) + col8 * 8;
        a_dst[it] = row * kLdsStride + col8 * 8;
    }
    uint32_t a_adj = 0;
    if (RAGGED) {
        const int col = (p.KT - 1) * 64 + (tid & 7) * 8;
        a_adj = col >= p.K ? static_cast<uint32_t>(col - (p.K - 8)) : 0u;
    }
    const int last = p.KT - 1;
    u32x4_t areg[D][A_LOADS];
    typename WB::Tile bq[D][FN];
    uint32_t bsz[D][FN][GPT];
    auto load_a = [&](int kt, u32x4_t* ar) {
        const half_t* base = p.A + kt * 64;
        const uint32_t d = (RAGGED && kt == last) ? a_adj : 0u;
#pragma unroll
        for (int it = 0; it < A_LOADS; ++it) ar[it] = *reinterpret_cast<const u32x4_t*>(base + (a_off[it] - d));
    };
    auto store_a = [&](int buf, const u32x4_t* ar) {
#pragma unroll
        for (int it = 0; it < A_LOADS; ++it) *reinterpret_cast<u32x4_t*>(&As[buf][a_dst[it]]) = ar[it];
    };
    auto load_b = [&](int kt, typename WB::Tile* q, uint32_t (*sz)[GPT]) {
#pragma unroll
        for (int fn = 0; fn < FN; ++fn) {
            q[fn] = WB::load(bbase[fn], kt, lane);
#pragma unroll
            for (int g = 0; g < GPT; ++g) {
                const int gi = (kt * 64 + g * 32) >> p.gshift;
                sz[fn][g] = (sbase[fn] + static_cast<size_t>(gi) * npad[fn])[l32];
            }
        }
    };

    // Ring slots: tile t's weights live in bq[t % D], tile t's activations in areg[t % D] until they are
    // parked in LDS buffer t % 3 during tile t-1.  The loop body is branch-free and runs over KT rounded up to
    // a multiple of D: loads past the last tile are clamped to it and the (at most D-1) surplus tiles get
    // scale|zero words of 0, so their weights dequantize to exactly 0 and add nothing.  Any branch around
    // the loads makes the compiler drain the whole load queue at every tile (its wait-count bookkeeping
    // merges the paths conservatively), which turns the ring back into a one-tile latency chain.
#pragma unroll
    for (int u = 0; u < D; ++u) {
        load_a(min(u, last), areg[u]);
        load_b(min(u, last), bq[u], bsz[u]);
    }
    store_a(0, areg[0]);
    load_a(min(D, last), areg[0]);
    __syncthreads();

    const int a_row0 = l32 * kLdsStride + lhi * 8;
    half8_t a[2][FM];
#pragma unroll
    for (int fm = 0; fm < FM; ++fm) a[0][fm] = *reinterpret_cast<const half8_t*>(&As[0][a_row0 + fm * 32 * kLdsStride]);
    int buf = 0;
    for (int kt0 = 0; kt0 < p.KT; kt0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int kt = kt0 + u;
            const int nbuf = buf == NBUF - 1 ? 0 : buf + 1;
            typename WB::SZ sz[FN][GPT];
#pragma unroll
            for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                for (int g = 0; g < GPT; ++g) sz[fn][g] = WB::expand(kt <= last ? bsz[u][fn][g] : 0u);
            const half_t* Ab = &As[buf][a_row0];
            const half_t* An = &As[nbuf][a_row0];
            half8_t bcur = WB::dequant(bq[u][0], 0, sz[0][0], magic);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (j == 1) {
                    // tile kt+1 becomes visible in LDS; three buffers make the write safe against waves still
                    // reading tile kt-1.  Its ring slot (u+1)%D then takes tile kt+1+D.
                    store_a(nbuf, areg[(u + 1) % D]);
                    load_a(min(kt + 1 + D, last), areg[(u + 1) % D]);
                    __syncthreads();
                }
#pragma unroll
                for (int fm = 0; fm < FM; ++fm)
                    a[(j + 1) & 1][fm] = *reinterpret_cast<const half8_t*>((j + 1 < 4 ? Ab + (j + 1) * 16 : An) + fm * 32 * kLdsStride);
#pragma unroll
                for (int fn = 0; fn < FN; ++fn) {
                    // the next fragment is dequantized while the matrix core works on the current one
                    const int fnn = fn + 1 < FN ? fn + 1 : 0;
                    const int jn = fn + 1 < FN ? j : j + 1;
                    half8_t bnext = bcur;
                    if (jn < 4) bnext = WB::dequant(bq[u][fnn], jn, sz[fnn][GPT == 2 ? (jn >> 1) : 0], magic);
#pragma unroll
                    for (int fm = 0; fm < FM; ++fm)
                        acc[fm][fn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[j & 1][fm], bcur, acc[fm][fn], 0, 0, 0);
                    bcur = bnext;
                }
            }
            load_b(min(kt + D, last), bq[u], bsz[u]);
            buf = nbuf;
        }
    }
    __syncthreads();     // every wave is done with the A tiles: the epilogue reuses the LDS

    store_tile<EPI, FM, FN>(p, acc, reinterpret_cast<float*>(smem) + wave * kSlabFloats, lane, m0, (tile_n * 4 + wave) * FN, M);
}

template <int BITS, int GPT, int EPI>
static hipError_t launch_epi(GemmDev& d, hipStream_t stream) {
    constexpr int FN = EPI == EPI_SWIGLU_F16 ? 2 : 1;
    constexpr int D = FN == 1 ? 4 : 3;      // ring depth: what the register budget of the variant holds without spilling
    d.tiles_m = (d.M_max + 63) / 64;
    d.tiles_n = (d.vf_total + 4 * FN - 1) / (4 * FN);
    const int blocks = ((d.tiles_n + 7) / 8) * 8 * d.tiles_m;
    if (blocks == 0) return hipSuccess;
    if (d.K % 64 != 0)
        hipLaunchKernelGGL((gemm_mid_kernel<BITS, FN, D, GPT, EPI, true>), dim3(blocks), dim3(256), 0, stream, d);
    else
        hipLaunchKernelGGL((gemm_mid_kernel<BITS, FN, D, GPT, EPI, false>), dim3(blocks), dim3(256), 0, stream, d);
    return hipGetLastError();
}

template <int BITS, int GPT>
static hipError_t launch_gpt(GemmDev& d, int epi, hipStream_t stream) {
    switch (epi) {
        case EPI_STORE_F16: return launch_epi<BITS, GPT, EPI_STORE_F16>(d, stream);
        case EPI_RESID_F32: return launch_epi<BITS, GPT, EPI_RESID_F32>(d, stream);
        case EPI_SWIGLU_F16: return launch_epi<BITS, GPT, EPI_SWIGLU_F16>(d, stream);
        default: return launch_epi<BITS, GPT, EPI_RESID_SCATTER>(d, stream);
    }
}

hipError_t launch_gemm_mid(GemmDev& d, int epilogue, hipStream_t stream) {
    if (d.bits == 3) {
        if (d.gshift == 5) return launch_gpt<3, 2>(d, epilogue, stream);
        return launch_gpt<3, 1>(d, epilogue, stream);
    }
    if (d.bits == 2) {
        if (d.gshift == 5) return launch_gpt<2, 2>(d, epilogue, stream);
        return launch_gpt<2, 1>(d, epilogue, stream);
    }
    if (d.gshift == 5) return launch_gpt<4, 2>(d, epilogue, stream);
    return launch_gpt<4, 1>(d, epilogue, stream);
}

}  // namespace qtale
