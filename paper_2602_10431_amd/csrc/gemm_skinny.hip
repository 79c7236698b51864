// Skinny W4A16 / W3A16 GEMM for decode steps: at most 64 executed rows, so the linears stream their weights once
// and the question is bandwidth and latency, not matrix-core throughput (Sec. 4.1 weights; the executed
// rows come from the gather of App. B.2).
//
// Shape of the work: C[M<=64][N] = A[M][K] x W'[N][K]^T.  The weights (N*K/2 bytes) dominate; A is at most
// 64 x K fp16 and stays in L2.  A k-loop with a barrier per 64-wide tile would be latency-bound
// (K/64 round trips), so here nothing synchronises inside the k-loop:
//   * a workgroup owns NFB consecutive 32-column fragments and ALL of K; its NW waves split K by
//     interleaving k-tiles (wave w takes tiles w, w+NW, ...), each wave keeping its own accumulators for
//     all NFB fragments, so its A registers are reused NFB times;
//   * per tile a wave issues NFB 16-byte (3-bit codes: 12-byte) weight loads, contiguous in the prepacked layout,
//     the scale/zero words and its A tile (row-contiguous loads, re-laid out through a wave-private LDS
//     region); the weights are prefetched four tiles ahead and the activations two;
//   * the K-split partial sums meet once, at the end: every wave writes its accumulators as a [64][cols]
//     fp32 slab into LDS, one barrier, and all threads add the NW slabs in wave order (deterministic)
//     while applying the same fused epilogues as the prefill kernel with row-contiguous accesses.
// MF = 1 (M <= 32) halves the A loads and MFMAs.
#include "gemm_common.h"

namespace qtale {

template <int BITS, int NFB, int NW, int MF, int GPT, int EPI, bool RAGGED>
__global__ void __launch_bounds__(NW * 64, (NW <= 4 ? 2 : 1))
gemm_skinny_kernel(GemmDev p) {
    using WB = WBits<BITS>;
    constexpr int NT = NW * 64;
    constexpr int CW = NFB * 32;                 // accumulator columns per wave
    constexpr int CSTR = CW + 4;                 // slab row stride (floats)
    constexpr int ROWS = MF * 32;
    constexpr int AD = (NW <= 8 && MF == 1) ? 2 : 1;   // activation tiles staged in LDS per wave (ring)
    constexpr int ASTR = 72;                     // halves per staged A row (64 + 8: conflict-free 16-byte reads)
    constexpr int kSlabBytes = NW * ROWS * CSTR * 4;
    constexpr int kStageBytes = NW * AD * ROWS * ASTR * 2;
    __shared__ __attribute__((aligned(16))) char smem[kSlabBytes > kStageBytes ? kSlabBytes : kStageBytes];
    float* slab = reinterpret_cast<float*>(smem);

    // Workgroup id -> (column tile, 64-row chunk).  With more than 64 rows the weights are streamed once per
    // chunk; ids are dealt round-robin to the 8 XCDs, so the chunks of one column tile are given ids 8 apart:
    // they run on the same XCD right after each other and the second one finds the weights in that L2.
    const int within = blockIdx.x % (8 * p.row_chunks);
    const int tile_n = (blockIdx.x / (8 * p.row_chunks)) * 8 + (within & 7);
    if (tile_n >= p.tiles_n) return;
    int row0, M;
    if (!gemm_chunk_rows(p, (within >> 3) * 64, ROWS, row0, M)) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    const uint32_t magic = dequant_magic();

    const char* bbase[NFB];
    const uint32_t* sbase[NFB];
    int npad[NFB];
#pragma unroll
    for (int fn = 0; fn < NFB; ++fn) {
        int vf = tile_n * NFB + fn;
        if (vf >= p.vf_total) vf = p.vf_total - 1;
        int mat, f;
        map_fragment<EPI>(p, vf, mat, f);
        bbase[fn] = reinterpret_cast<const char*>(p.codes[mat]) + static_cast<size_t>(f) * p.KT * (64 * WB::kLaneBytes);
        sbase[fn] = p.sz[mat] + f * 32;
        npad[fn] = p.npad[mat];
    }

    float16_t acc[MF][NFB];
#pragma unroll
    for (int mf = 0; mf < MF; ++mf)
#pragma unroll
        for (int fn = 0; fn < NFB; ++fn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mf][fn][r] = 0.0f;

    // Activations: a wave fetches its k-tile of A (ROWS x 64 halves) with row-contiguous 16-byte loads (8
    // lanes per 128-byte row segment, so every cache line is consumed by the instruction that fetched it),
    // parks it in a wave-private LDS region and reads it back in MFMA operand order.  Reading the operand
    // layout straight from global memory touches each line with four different instructions and, with
    // 16 tiles in flight per CU, thrashes the 32 KB L1: that version moved four times the bytes.
    constexpr int A_LD = ROWS / 8;                   // 16-byte loads per lane per tile
    uint32_t a_off[A_LD];
#pragma unroll
    for (int it = 0; it < A_LD; ++it)
        a_off[it] = static_cast<uint32_t>(min(it * 8 + (lane >> 3), M - 1)) * static_cast<uint32_t>(p.K) + (lane & 7) * 8;
    half_t* stage_base = reinterpret_cast<half_t*>(smem) + wave * (AD * ROWS * ASTR);
    const int st_w = (lane >> 3) * ASTR + (lane & 7) * 8;          // where this lane parks its chunk (+ it*8 rows)
    const int st_r = l32 * ASTR + lhi * 8;                          // where it reads operand (mf, j) from

    // Wave w owns tiles w, w + NW, ...  Weights come from HBM (long latency, 5 registers per fragment and
    // tile) and are prefetched BD tiles ahead; activations come from L2 and are prefetched AD tiles ahead
    // in registers.  Loads past the wave's last tile are clamped to it (harmless, never consumed) so that
    // the load order in the loop is unconditional.
    constexpr int BD = NW <= 8 ? 4 : 2;           // weight tiles in flight per wave
    typename WB::Tile bq[BD][NFB];
    uint32_t bsz[BD][NFB][GPT];
    u32x4_t areg[AD][A_LD];
    auto fetch_b = [&](int kt, typename WB::Tile* q, uint32_t (*sz)[GPT]) {
#pragma unroll
        for (int fn = 0; fn < NFB; ++fn) {
            q[fn] = WB::load(bbase[fn], kt, lane);
#pragma unroll
            for (int g = 0; g < GPT; ++g) {
                const int gi = (kt * 64 + g * 32) >> p.gshift;
                sz[fn][g] = (sbase[fn] + static_cast<size_t>(gi) * npad[fn])[l32];
            }
        }
    };
    auto fetch_a = [&](int kt, u32x4_t* ar) {
        const half_t* base = p.A + static_cast<size_t>(row0) * p.K + kt * 64;
        uint32_t shift = 0;
        if (RAGGED) {                               // chunks starting at or beyond K read the row's last
            const int col = kt * 64 + (lane & 7) * 8;           // valid chunk: the weights there are 0
            shift = col >= p.K ? static_cast<uint32_t>(col - (p.K - 8)) : 0u;
        }
#pragma unroll
        for (int it = 0; it < A_LD; ++it) ar[it] = *reinterpret_cast<const u32x4_t*>(base + (a_off[it] - shift));
    };
    auto park_a = [&](const u32x4_t* ar, int slot) {
        half_t* dst = stage_base + slot * (ROWS * ASTR) + st_w;
#pragma unroll
        for (int it = 0; it < A_LD; ++it) *reinterpret_cast<u32x4_t*>(dst + it * 8 * ASTR) = ar[it];
    };
    auto compute = [&](const typename WB::Tile* q, const uint32_t (*szr)[GPT], int slot) {
        const half_t* src = stage_base + slot * (ROWS * ASTR) + st_r;
        typename WB::SZ sz[NFB][GPT];
#pragma unroll
        for (int fn = 0; fn < NFB; ++fn)
#pragma unroll
            for (int g = 0; g < GPT; ++g) sz[fn][g] = WB::expand(szr[fn][g]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            half8_t a[MF];
#pragma unroll
            for (int mf = 0; mf < MF; ++mf) a[mf] = *reinterpret_cast<const half8_t*>(src + mf * 32 * ASTR + j * 16);
#pragma unroll
            for (int fn = 0; fn < NFB; ++fn) {
                const half8_t b = WB::dequant(q[fn], j, sz[fn][GPT == 2 ? (j >> 1) : 0], magic);
#pragma unroll
                for (int mf = 0; mf < MF; ++mf)
                    acc[mf][fn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[mf], b, acc[mf][fn], 0, 0, 0);
            }
        }
    };

    const int n_mine = wave < p.KT ? (p.KT - wave + NW - 1) / NW : 0;     // tiles of this wave
    if (n_mine > 0) {
        const int last = wave + (n_mine - 1) * NW;
#pragma unroll
        for (int u = 0; u < BD; ++u) fetch_b(min(wave + u * NW, last), bq[u], bsz[u]);
#pragma unroll
        for (int u = 0; u < AD; ++u) fetch_a(min(wave + u * NW, last), areg[u]);
        for (int i0 = 0; i0 < n_mine; i0 += BD) {
#pragma unroll
            for (int u = 0; u < BD; ++u) {
                const int i = i0 + u;
                // the LDS slot of tile i was last read by tile i - AD of this same wave (LDS ops of a wave
                // complete in order), so parking needs no barrier
                park_a(areg[u % AD], u % AD);
                fetch_a(min(wave + (i + AD) * NW, last), areg[u % AD]);
                if (i < n_mine) compute(bq[u], bsz[u], u % AD);
                fetch_b(min(wave + (i + BD) * NW, last), bq[u], bsz[u]);
            }
        }
    }
    __syncthreads();     // the slabs below overlay the A staging regions of other waves

    // ---- meet: slabs into LDS, one barrier, ordered sum + epilogue ----------------------------------
    float* mine = slab + wave * (ROWS * CSTR);
#pragma unroll
    for (int mf = 0; mf < MF; ++mf)
#pragma unroll
        for (int fn = 0; fn < NFB; ++fn)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                mine[(mf * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3)) * CSTR + fn * 32 + l32] = acc[mf][fn][r];
    __syncthreads();

    constexpr int NFO = EPI == EPI_SWIGLU_F16 ? NFB / 2 : NFB;   // output fragments of the workgroup
    constexpr int CWO = NFO * 32;
    constexpr int LPR = CWO / 4;                                 // lanes per output row (4 columns each)
    constexpr int RPP = NT / LPR;                                // rows per pass
    const int c4 = (tid % LPR) * 4;
    const int fo = c4 >> 5;
    int o_vf = tile_n * NFB + (EPI == EPI_SWIGLU_F16 ? 2 * fo : fo);
    const bool o_valid = o_vf < p.vf_total;
    int o_mat, o_f;
    map_fragment<EPI>(p, o_valid ? o_vf : p.vf_total - 1, o_mat, o_f);
    const int o_ncol = o_f * 32 + (c4 & 31);
    const bool col_ok = o_valid && o_ncol < p.N[o_mat];
    const int col = (EPI == EPI_SWIGLU_F16 ? 0 : p.colbase[o_mat]) + o_ncol;
    // slab column of the lane's first value (SwiGLU: gate fragment 2*fo, up fragment 2*fo+1)
    const int sc = EPI == EPI_SWIGLU_F16 ? (2 * fo) * 32 + (c4 & 31) : c4;

    for (int lrow = tid / LPR; lrow < ROWS; lrow += RPP) {
        if (!col_ok || lrow >= M) continue;
        const int row = row0 + lrow;                 // row of the whole activation / output matrix
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f), u = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float* s = slab + w * (ROWS * CSTR) + lrow * CSTR + sc;
            const float4 t = *reinterpret_cast<const float4*>(s);
            v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
            if (EPI == EPI_SWIGLU_F16) {
                const float4 t2 = *reinterpret_cast<const float4*>(s + 32);
                u.x += t2.x; u.y += t2.y; u.z += t2.z; u.w += t2.w;
            }
        }
        if (EPI == EPI_SWIGLU_F16) {
            v.x = silu_f(v.x) * u.x; v.y = silu_f(v.y) * u.y; v.z = silu_f(v.z) * u.z; v.w = silu_f(v.w) * u.w;
        }
        if (EPI == EPI_STORE_F16 || EPI == EPI_SWIGLU_F16) {
            uint2 o;
            o.x = static_cast<uint32_t>(float_to_half_bits(v.x)) | (static_cast<uint32_t>(float_to_half_bits(v.y)) << 16);
            o.y = static_cast<uint32_t>(float_to_half_bits(v.z)) | (static_cast<uint32_t>(float_to_half_bits(v.w)) << 16);
            *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(p.out) + static_cast<size_t>(row) * p.ldo + col) = o;
        } else if (EPI == EPI_RESID_F32) {
            const int t = p.idx[row];
            const uint2 xr = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(p.resid) + static_cast<size_t>(t) * p.ldo + col);
            float4 o;
            o.x = act_to_float(static_cast<uint16_t>(xr.x & 0xffffu), p.bf16) + v.x;
            o.y = act_to_float(static_cast<uint16_t>(xr.x >> 16), p.bf16) + v.y;
            o.z = act_to_float(static_cast<uint16_t>(xr.y & 0xffffu), p.bf16) + v.z;
            o.w = act_to_float(static_cast<uint16_t>(xr.y >> 16), p.bf16) + v.w;
            *reinterpret_cast<float4*>(reinterpret_cast<float*>(p.out) + static_cast<size_t>(row) * p.ldo + col) = o;
        } else {
            const int t = p.idx[row];
            const float4 res = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(p.resid) + static_cast<size_t>(row) * p.ldo + col);
            uint2 o;
            o.x = static_cast<uint32_t>(float_to_act(res.x + v.x, p.bf16)) | (static_cast<uint32_t>(float_to_act(res.y + v.y, p.bf16)) << 16);
            o.y = static_cast<uint32_t>(float_to_act(res.z + v.z, p.bf16)) | (static_cast<uint32_t>(float_to_act(res.w + v.w, p.bf16)) << 16);
            *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(p.out) + static_cast<size_t>(t) * p.ldo + col) = o;
        }
    }
}

template <int BITS, int NFB, int NW, int MF, int GPT, int EPI>
static hipError_t launch_one(GemmDev& d, hipStream_t stream) {
    d.tiles_n = (d.vf_total + NFB - 1) / NFB;
    if (d.tiles_n == 0) return hipSuccess;
    d.row_chunks = (d.M_max + 63) / 64;
    const int blocks = ((d.tiles_n + 7) / 8) * 8 * d.row_chunks;
    if (d.K % 64 != 0)
        hipLaunchKernelGGL((gemm_skinny_kernel<BITS, NFB, NW, MF, GPT, EPI, true>), dim3(blocks), dim3(NW * 64), 0, stream, d);
    else
        hipLaunchKernelGGL((gemm_skinny_kernel<BITS, NFB, NW, MF, GPT, EPI, false>), dim3(blocks), dim3(NW * 64), 0, stream, d);
    return hipGetLastError();
}

template <int BITS, int GPT, int EPI>
static hipError_t launch_shape(GemmDev& d, hipStream_t stream) {
    // Pick the split so that one round of workgroups covers the chip: very wide outputs (gate/up) use four
    // waves per workgroup and two workgroups per CU, wide ones eight waves, narrow ones (few fragments)
    // one fragment per workgroup and 16 K-slices so that more CUs take part.
    if (EPI == EPI_SWIGLU_F16 || d.vf_total >= 512) {
        if (d.M_max <= 32) return launch_one<BITS, 2, 4, 1, GPT, EPI>(d, stream);
        return launch_one<BITS, 2, 4, 2, GPT, EPI>(d, stream);
    }
    if (d.vf_total >= 256) {
        if (d.M_max <= 32) return launch_one<BITS, 2, 8, 1, GPT, EPI>(d, stream);
        return launch_one<BITS, 2, 8, 2, GPT, EPI>(d, stream);
    }
    if constexpr (EPI != EPI_SWIGLU_F16) {
        if (d.M_max <= 32) return launch_one<BITS, 1, 16, 1, GPT, EPI>(d, stream);
        return launch_one<BITS, 1, 16, 2, GPT, EPI>(d, stream);
    }
    return hipErrorInvalidValue;       // SwiGLU always takes the first branch
}

template <int BITS, int GPT>
static hipError_t launch_gpt(GemmDev& d, int epi, hipStream_t stream) {
    switch (epi) {
        case EPI_STORE_F16: return launch_shape<BITS, GPT, EPI_STORE_F16>(d, stream);
        case EPI_RESID_F32: return launch_shape<BITS, GPT, EPI_RESID_F32>(d, stream);
        case EPI_SWIGLU_F16: return launch_shape<BITS, GPT, EPI_SWIGLU_F16>(d, stream);
        default: return launch_shape<BITS, GPT, EPI_RESID_SCATTER>(d, stream);
    }
}

hipError_t launch_gemm_skinny(GemmDev& d, int epilogue, hipStream_t stream) {
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
