// W4A16 / W3A16 / W2A16 GEMM for decode steps (at most 64 executed rows): C[M][N] = A[M][K] x W'[N][K]^T with the
// weights streamed once (Sec. 4.1 weights; the rows are the executed tokens gathered per App. B.2).
//
// What bounds this shape on gfx950 is not the matrix cores and not HBM alone but how much of each a CU can
// overlap: a wave that owns a whole 64-row x 64-column tile is a long serial chain (activation loads, LDS round
// trip, dequantisation, MFMAs that block the wave's own issue) with too many registers for more than one or two
// waves per SIMD, and every CU has to pull the 64 x K activation panel through its 64 B/clk vector-memory path
// once per column block it serves.  So here
//   * a wave owns ONE 32-column weight fragment and a quarter of the workgroup's k-tiles (32 accumulator
//     registers), which leaves room for three to four waves per SIMD: their loads, dequantisation and MFMAs overlap;
//   * the NWN waves that work on the same k-tile share its activation tile: they fetch it together (a few 16-byte
//     chunks per lane), park it in LDS and all read their MFMA operands from there, so a CU fetches the activation
//     panel once per NWN fragments;
//   * workgroup = NWN fragments x 4 k-slices (waves wn + NWN * wk), all of K unless the output is so narrow that
//     column blocks alone cannot fill the chip: then K is also cut across workgroups and every workgroup writes an
//     fp32 partial tile that the consumer kernel adds in slice order (no atomics, no fences: deterministic);
//   * weights and activations of D rounds are in flight per wave (register rings, the loop is unrolled by D);
//   * gate/up: a fragment is made of 16 gate rows and 16 up rows of the same output columns, so SiLU(gate)*up
//     needs no second fragment and the column blocks can be sized to one workgroup per CU;
//   * the k-slices meet once in LDS (ordered sum) and the epilogue writes row-contiguous pieces.
#include <algorithm>

#include "gemm_common.h"

namespace qtale {

constexpr int kDecNWK = 4;          // k-slices (waves along K) per workgroup

template <int BITS, int NWN, int MF, int GPT>
__global__ void __launch_bounds__(NWN * kDecNWK * 64, 1)
gemm_decode_kernel(GemmDev p) {
    using WB = WBits<BITS>;
    constexpr int NWK = kDecNWK;
    constexpr int NW = NWN * NWK;
    constexpr int ROWS = MF * 32;
    constexpr int TEAM = NWN * 64;                               // lanes that fetch one activation tile together
    constexpr int A_CH = ROWS * 8;                               // 16-byte chunks of a ROWS x 64 tile
    constexpr int A_LD = (A_CH + TEAM - 1) / TEAM;               // chunks per lane
    constexpr int D = 3;                                         // rounds in flight
    constexpr int kTileHalves = ROWS * kLdsStride;
    constexpr int kABytes = 2 * NWK * kTileHalves * 2;           // two buffers x NWK tiles
    constexpr int SSTR = 36;                                     // slab row stride (floats)
    constexpr int kSlabBytes = NW * ROWS * SSTR * 4;             // every wave's accumulators
    __shared__ __attribute__((aligned(16))) char smem[kABytes > kSlabBytes ? kABytes : kSlabBytes];
    half_t* As = reinterpret_cast<half_t*>(smem);

    // workgroup -> (column block, 64-row chunk, k-part).  Ids are dealt round-robin to the 8 XCDs: the row chunks
    // of one column block get ids 8 apart, so they stream the same weights through the same L2.
    const int within = blockIdx.x % (8 * p.row_chunks);
    const int tile_n = (blockIdx.x / (8 * p.row_chunks)) * 8 + (within & 7);
    const int ks = blockIdx.y;
    if (tile_n >= p.tiles_n) return;
    int row0, M;
    if (!gemm_chunk_rows(p, (within >> 3) * 64, ROWS, row0, M)) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave % NWN, wk = wave / NWN;
    const int l32 = lane & 31, lhi = lane >> 5;
    const uint32_t magic = dequant_magic();
    const bool swiglu = p.epi_rt == EPI_SWIGLU_F16;

    // k-tiles of this workgroup: part ks of KT (parts differ by at most one tile); slice wk takes every NWK-th
    const int kt_lo = static_cast<int>(static_cast<long>(p.KT) * ks / p.ksplit);
    const int kt_hi = static_cast<int>(static_cast<long>(p.KT) * (ks + 1) / p.ksplit);
    const int n_rounds = (kt_hi - kt_lo + NWK - 1) / NWK;

    // ---- this lane's weight row: per-lane pointers (gate/up fragments mix two matrices) -----------------
    const char* bptr;
    const uint32_t* sptr;
    int npad;
    {
        int vf = tile_n * NWN + wn;
        if (vf >= p.vf_total) vf = p.vf_total - 1;               // edge block: recompute the last fragment, never stored
        int mat = 0, f = vf, lane_row = l32;
        if (swiglu) {                                            // rows 16 vf .. 16 vf + 15 of gate (lanes 0-15) and of up (16-31)
            mat = l32 >> 4;
            f = vf >> 1;
            lane_row = ((vf & 1) << 4) | (l32 & 15);
        } else {
            if (p.n_w > 1 && f >= p.NF[0]) { f -= p.NF[0]; mat = 1; }
            if (p.n_w > 2 && mat == 1 && f >= p.NF[1]) { f -= p.NF[1]; mat = 2; }
        }
        const void* cbase = mat == 0 ? p.codes[0] : mat == 1 ? p.codes[1] : p.codes[2];
        const uint32_t* zbase = mat == 0 ? p.sz[0] : mat == 1 ? p.sz[1] : p.sz[2];
        npad = mat == 0 ? p.npad[0] : mat == 1 ? p.npad[1] : p.npad[2];
        bptr = reinterpret_cast<const char*>(cbase) + (static_cast<size_t>(f) * p.KT * 64 + (lhi * 32 + lane_row)) * WB::kLaneBytes;
        sptr = zbase + f * 32 + lane_row;
    }

    float16_t acc[MF];
#pragma unroll
    for (int mf = 0; mf < MF; ++mf)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mf][r] = 0.0f;

    // ---- activation tile of this wave's k-slice: fetched by the slice's NWN waves together ----------------
    const int tl = wn * 64 + lane;                               // lane index inside the team
    uint32_t a_off[A_LD];
    int a_dst[A_LD];
    bool a_ok[A_LD];
#pragma unroll
    for (int it = 0; it < A_LD; ++it) {
        const int c = it * TEAM + tl;
        a_ok[it] = c < A_CH;
        const int row = (c < A_CH ? c : A_CH - 1) >> 3, col8 = c & 7;
        a_off[it] = static_cast<uint32_t>(row0 + min(row, M - 1)) * static_cast<uint32_t>(p.K) + col8 * 8;
        a_dst[it] = row * kLdsStride + col8 * 8;
    }
    // round r works on tile kt_lo + r * NWK + wk of this slice; rounds past the slice's last tile are clamped to it
    // and get a scale|zero word of 0 (their weights dequantize to exactly 0), so the load order never branches
    const int kt_last = kt_hi - 1;
    auto tile_of = [&](int r) { return min(kt_lo + r * NWK + wk, kt_last); };
    u32x4_t areg[D][A_LD];
    auto load_a = [&](int r, u32x4_t* ar) {
        const int kt = tile_of(r);
        const half_t* base = p.A + kt * 64;
        // chunks that start at or beyond K (K not a multiple of 64) read the row's last valid chunk: the
        // weights there are the zero-point (dequantize to 0)
        const int col = kt * 64 + (tl & 7) * 8;
        const uint32_t shift = col >= p.K ? static_cast<uint32_t>(col - (p.K - 8)) : 0u;
#pragma unroll
        for (int it = 0; it < A_LD; ++it) ar[it] = *reinterpret_cast<const u32x4_t*>(base + (a_off[it] - shift));
    };
    auto store_a = [&](int buf, const u32x4_t* ar) {
        half_t* dst = As + (buf * NWK + wk) * kTileHalves;
#pragma unroll
        for (int it = 0; it < A_LD; ++it)
            if ((A_CH % TEAM) == 0 || a_ok[it]) *reinterpret_cast<u32x4_t*>(dst + a_dst[it]) = ar[it];
    };
    auto load_b = [&](int r, typename WB::Tile& q, uint32_t* sz) {
        const int kt = tile_of(r);
        q = WB::load_lane(bptr + static_cast<size_t>(kt) * (64 * WB::kLaneBytes));
#pragma unroll
        for (int g = 0; g < GPT; ++g) {
            const int gi = (kt * 64 + g * 32) >> p.gshift;
            sz[g] = sptr[static_cast<size_t>(gi) * npad];
        }
    };
    const int a_rd = l32 * kLdsStride + lhi * 8;
    auto compute = [&](int r, int buf, const typename WB::Tile& q, const uint32_t* szr) {
        const bool live = kt_lo + r * NWK + wk <= kt_last;
        typename WB::SZ sz[GPT];
#pragma unroll
        for (int g = 0; g < GPT; ++g) sz[g] = WB::expand(live ? szr[g] : 0u);
        const half_t* src = As + (buf * NWK + wk) * kTileHalves + a_rd;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            half8_t a[MF];
#pragma unroll
            for (int mf = 0; mf < MF; ++mf) a[mf] = *reinterpret_cast<const half8_t*>(src + mf * 32 * kLdsStride + j * 16);
            const half8_t b = WB::dequant(q, j, sz[GPT == 2 ? (j >> 1) : 0], magic);
#pragma unroll
            for (int mf = 0; mf < MF; ++mf) acc[mf] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[mf], b, acc[mf], 0, 0, 0);
        }
    };

    // Round r is computed from LDS buffer r & 1.  While it is, the activations of round r + 1 (fetched D rounds
    // ago) are parked in the other buffer and the fetches of round r + 1 + D and r + D are issued; the barrier at
    // the end of the round makes the parked tile visible and guarantees nobody still reads the buffer that the
    // next round overwrites.
    typename WB::Tile bq[D];
    uint32_t bsz[D][GPT];
#pragma unroll
    for (int u = 0; u < D; ++u) {
        load_a(u, areg[u]);
        load_b(u, bq[u], bsz[u]);
    }
    store_a(0, areg[0]);
    load_a(D, areg[0]);
    __syncthreads();
    for (int r0 = 0; r0 < n_rounds; r0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int r = r0 + u;
            store_a((r + 1) & 1, areg[(u + 1) % D]);
            load_a(r + 1 + D, areg[(u + 1) % D]);
            if (r < n_rounds) compute(r, r & 1, bq[u], bsz[u]);
            load_b(r + D, bq[u], bsz[u]);
            __syncthreads();
        }
    }

    // ---- meet: the NWK k-slices of every fragment are added in slice order -----------------------------------
    float* slab = reinterpret_cast<float*>(smem);
    const int cw = swiglu ? 16 : 32;                             // output columns per fragment
    const int lpr = NWN * (cw >> 2);                             // lanes per output row (4 columns each)
    const int item_row = tid / lpr, item_q = tid % lpr;
    const int wn_c = item_q / (cw >> 2), c4 = (item_q % (cw >> 2)) * 4;
    const bool item_ok = item_row < 32;
    int o_vf = tile_n * NWN + wn_c;
    const bool vf_ok = o_vf < p.vf_total;
    if (!vf_ok) o_vf = p.vf_total - 1;
    int o_mat = 0, o_f = o_vf;
    if (!swiglu) {
        if (p.n_w > 1 && o_f >= p.NF[0]) { o_f -= p.NF[0]; o_mat = 1; }
        if (p.n_w > 2 && o_mat == 1 && o_f >= p.NF[1]) { o_f -= p.NF[1]; o_mat = 2; }
    }
    const int o_ncol = (swiglu ? o_vf * 16 : o_f * 32) + c4;
    const int o_n = o_mat == 0 ? p.N[0] : o_mat == 1 ? p.N[1] : p.N[2];
    const bool col_ok = item_ok && vf_ok && o_ncol < o_n;        // N % 4 == 0: the 4 columns are all in or all out
    const int col = (swiglu ? 0 : (o_mat == 0 ? p.colbase[0] : o_mat == 1 ? p.colbase[1] : p.colbase[2])) + o_ncol;
    {
        float* mine = slab + wave * (ROWS * SSTR);
#pragma unroll
        for (int mf = 0; mf < MF; ++mf)
#pragma unroll
            for (int r = 0; r < 16; ++r) mine[(mf * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3)) * SSTR + l32] = acc[mf][r];
    }
    __syncthreads();
#pragma unroll
    for (int mf = 0; mf < MF; ++mf) {
        const int lrow = mf * 32 + item_row;
        if (col_ok && lrow < M) {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f), u = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int k = 0; k < NWK; ++k) {
                const float* s = slab + (k * NWN + wn_c) * (ROWS * SSTR) + lrow * SSTR + c4;
                const float4 t = *reinterpret_cast<const float4*>(s);
                v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
                if (swiglu) {
                    const float4 t2 = *reinterpret_cast<const float4*>(s + 16);
                    u.x += t2.x; u.y += t2.y; u.z += t2.z; u.w += t2.w;
                }
            }
            const int row = row0 + lrow;
            if (p.epi_rt == EPI_PARTIAL_F32) {
                float* dst = reinterpret_cast<float*>(p.out) + (static_cast<size_t>(ks) * p.M_max + row) * p.ldo + col;
                *reinterpret_cast<float4*>(dst) = v;
            } else {
                if (swiglu) {
                    v.x = silu_f(v.x) * u.x; v.y = silu_f(v.y) * u.y; v.z = silu_f(v.z) * u.z; v.w = silu_f(v.w) * u.w;
                }
                uint2 o;
                o.x = static_cast<uint32_t>(float_to_half_bits(v.x)) | (static_cast<uint32_t>(float_to_half_bits(v.y)) << 16);
                o.y = static_cast<uint32_t>(float_to_half_bits(v.z)) | (static_cast<uint32_t>(float_to_half_bits(v.w)) << 16);
                *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(p.out) + static_cast<size_t>(row) * p.ldo + col) = o;
            }
        }
    }
}

template <int BITS, int NWN, int MF, int GPT>
static hipError_t launch_one(const GemmDev& d, hipStream_t stream) {
    const dim3 grid(((d.tiles_n + 7) / 8) * 8 * d.row_chunks, d.ksplit), block(NWN * kDecNWK * 64);
    hipLaunchKernelGGL((gemm_decode_kernel<BITS, NWN, MF, GPT>), grid, block, 0, stream, d);
    return hipGetLastError();
}

template <int BITS, int GPT>
static hipError_t launch_nwn(const GemmDev& d, int nwn, hipStream_t stream) {
    const bool small = d.M_max <= 32;
    switch (nwn) {
        case 2: return small ? launch_one<BITS, 2, 1, GPT>(d, stream) : launch_one<BITS, 2, 2, GPT>(d, stream);
        case 3: return small ? launch_one<BITS, 3, 1, GPT>(d, stream) : launch_one<BITS, 3, 2, GPT>(d, stream);
        default: return small ? launch_one<BITS, 4, 1, GPT>(d, stream) : launch_one<BITS, 4, 2, GPT>(d, stream);
    }
}

// CUs of the current device (queried once per device).
static int decode_cus() {
    static int cus[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cus[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cus[dev] = n;
    }
    return cus[dev];
}

// Fragments per workgroup and k-parts.  One workgroup per CU is the aim: take the narrowest column block (2, 3 or
// 4 fragments) whose blocks do not outnumber the CUs, and when even the narrowest leaves most CUs idle and the
// caller can take partial sums (split_max > 1), cut K across workgroups.
int gemm_decode_plan(const GemmDev& d, int epilogue, int split_max, int* nwn_out) {
    const int cus = decode_cus();
    const int chunks = (d.M_max + 63) / 64;
    const int n_frag = epilogue == EPI_SWIGLU_F16 ? (d.N[0] + 15) / 16 : d.vf_total;
    int nwn = 4;
    for (int c = 2; c <= 4; ++c)
        if (((n_frag + c - 1) / c) * chunks <= cus) { nwn = c; break; }
    int split = 1;
    if (split_max > 1) {
        nwn = 2;
        const int blocks = ((n_frag + 1) / 2) * chunks;
        split = std::max(1, std::min(split_max, cus / std::max(blocks, 1)));
        split = std::min(split, std::max(1, d.KT / kDecNWK));    // every part keeps at least one round of real tiles
    }
    *nwn_out = nwn;
    return split;
}

hipError_t launch_gemm_decode(GemmDev& d, int epilogue, int nwn, int split, hipStream_t stream) {
    const int n_frag = epilogue == EPI_SWIGLU_F16 ? (d.N[0] + 15) / 16 : d.vf_total;
    d.vf_total = n_frag;
    d.tiles_n = (n_frag + nwn - 1) / nwn;
    if (d.tiles_n == 0) return hipSuccess;
    d.row_chunks = (d.M_max + 63) / 64;
    d.ksplit = split;
    d.epi_rt = epilogue;
    if (d.bits == 3) return d.gshift == 5 ? launch_nwn<3, 2>(d, nwn, stream) : launch_nwn<3, 1>(d, nwn, stream);
    if (d.bits == 2) return d.gshift == 5 ? launch_nwn<2, 2>(d, nwn, stream) : launch_nwn<2, 1>(d, nwn, stream);
    return d.gshift == 5 ? launch_nwn<4, 2>(d, nwn, stream) : launch_nwn<4, 1>(d, nwn, stream);
}

}  // namespace qtale
