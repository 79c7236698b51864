// W4A16 / W3A16 GEMM for the layer's linears on the compacted tokens: C[M][N] = A[M][K] (fp16) x W'[N][K]^T,
// W' = (code - zero) * scale per group of the input dimension (Sec. 4.1 weight-only group quantization,
// 4-bit and 3-bit codes).
//
// Design for gfx950 (64-wide waves, v_mfma_f32_32x32x16_f16, 160 KB LDS):
//   * Weights are the B operand.  In the prepacked layout one 16-byte load gives a lane the 4 x 8 codes
//     of its row n = lane%32 for the four 16-wide k-steps of a 64-wide k-tile, already in operand order,
//     so weights go HBM/L2 -> VGPR -> (dequantize) -> MFMA and never touch LDS.
//   * Dequantisation is packed fp16: OR-ing a nibble into 0x6400 gives the fp16 value 1024 + c (low
//     nibble position) or 1024 + 16 c (next position); (1024+c) - (1024+z) and (1024+16c)/16 - (64+z)
//     are exact, one multiply by the scale rounds once.  13 VALU ops per 8 weights.
//   * Activations are the A operand, staged global -> VGPR -> LDS (row stride 72 halves: conflict-free
//     16-byte reads) through three LDS buffers with one barrier per k-tile placed in the middle of the
//     tile, so a wave's MFMA stream never stops at a tile boundary (see the pipeline comment below).
//   * Workgroup tile 128(M) x 256(N), 4 waves of 128 x 64, two workgroups resident per CU: the second
//     workgroup's waves fill the issue slots a wave loses while its own MFMA is in flight.
//   * Epilogues fuse what follows the linear: fp16 store (q|k|v), residual add from the gathered rows
//     of x into an fp32 h (o-proj), SiLU(gate)*up (MLP), residual add + scatter back into x (down-proj).
//     The accumulators are transposed through LDS so that every global access is row-contiguous.
#include <algorithm>
#include <type_traits>

#include "gemm_common.h"

namespace qtale {

template <int BITS, int WM, int WN, int FM, int FN, int GPT, int EPI, int OCC, bool RAGGED>
__global__ void __launch_bounds__(WM * WN * 64, OCC)
gemm_w4a16_kernel(GemmDev p) {
    using WB = WBits<BITS>;
    constexpr int NT = WM * WN * 64;
    constexpr int BM = WM * FM * 32;
    constexpr int A_LOADS = (BM * 8) / NT;
    static_assert((BM * 8) % NT == 0, "A tile must split evenly over the threads");
    static_assert(EPI != EPI_SWIGLU_F16 || (FN % 2) == 0, "gate/up fragments come in pairs");

    constexpr int NBUF = 3;                                     // LDS buffers of the A tile
    constexpr int kABytes = NBUF * BM * kLdsStride * 2;
    constexpr int kCBytes = WM * WN * 32 * ((EPI == EPI_SWIGLU_F16 ? FN / 2 : FN) * 32 + 8) * 4;
    __shared__ __attribute__((aligned(16))) char smem[kABytes > kCBytes ? kABytes : kCBytes];
    half_t (*As)[BM * kLdsStride] = reinterpret_cast<half_t (*)[BM * kLdsStride]>(smem);

    // One workgroup per tile.  In ratio mode the host knows the row count and sizes the grid for it; in threshold
    // mode M is a device-side count and the grid covers the host bound: tile ids run down the LIVE row tiles of
    // one column panel first (tile % live_m), so the ids beyond the live tiles form the end of the grid and their
    // workgroups leave at once.  (Measured on the 7B-shaped stack at 5-52 % executed rows: 1-7 % faster than a
    // chip-sized grid of workgroups that walk the live tiles, whose pipeline restarts at every tile.)
    int M = p.count ? min(*p.count, p.M_max) : p.M_max;
    if (p.tail == 1) M -= gemm_tail_rows(M, p.tail_tiles_n, p.tail_slots);                    // those rows go to a small-row launch
    const int live_m = (M + BM - 1) / BM;
    const int n_tiles = live_m * p.tiles_n;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform: lives in an SGPR
    const int wm = wave % WM;
    const int wn = wave / WM;
    const int l32 = lane & 31;
    const int lhi = lane >> 5;
    const uint32_t magic = dequant_magic();

    const int tile = blockIdx.x;
    if (tile >= n_tiles) return;
    const int tile_m = tile % live_m;
    const int tile_n = tile / live_m;
    const int m0 = tile_m * BM;

    // ---- which weight fragments this wave owns (all wave-uniform -> scalar base addresses) ------
    const char* bbase[FN];
    const uint32_t* sbase[FN];
    int npad[FN];
#pragma unroll
    for (int fn = 0; fn < FN; ++fn) {
        int vf = (tile_n * WN + wn) * FN + fn;
        if (vf >= p.vf_total) vf = p.vf_total - 1;     // edge tile: recompute the last fragment, never stored
        int mat, f;
        if (EPI == EPI_SWIGLU_F16) {
            mat = vf & 1;
            f = vf >> 1;
        } else {
            mat = 0;
            f = vf;
            if (p.n_w > 1 && f >= p.NF[0]) { f -= p.NF[0]; mat = 1; }
            if (p.n_w > 2 && mat == 1 && f >= p.NF[1]) { f -= p.NF[1]; mat = 2; }
        }
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

    // ---- A tile: global -> registers -> LDS ------------------------------------------------------
    // Every global address is (uniform base advanced per k-tile) + (per-lane offset fixed for the whole
    // kernel).  When K is not a multiple of 64 (RAGGED) the chunks of the last tile that start at or
    // beyond K are redirected to the row's last valid chunk: the weights there dequantize to exactly 0
    // (prepack pads with the zero-point), so any finite activation contributes nothing.
    u32x4_t areg[A_LOADS];
    uint32_t a_off[A_LOADS];        // element offset of this thread's chunk inside A (rows clamped to M-1)
    int a_dst[A_LOADS];
#pragma unroll
    for (int it = 0; it < A_LOADS; ++it) {
        const int c = it * NT + tid;
        const int row = c >> 3, col8 = c & 7;
        const int gr = min(m0 + row, M - 1);
        a_off[it] = static_cast<uint32_t>(gr) * static_cast<uint32_t>(p.K) + col8 * 8;
        a_dst[it] = row * kLdsStride + col8 * 8;
    }
    uint32_t a_adj = 0;             // RAGGED: how far this thread's chunk overshoots K in the last tile
    if (RAGGED) {
        const int col = (p.KT - 1) * 64 + (tid & 7) * 8;      // NT % 8 == 0: same column chunk for every `it`
        a_adj = col >= p.K ? static_cast<uint32_t>(col - (p.K - 8)) : 0u;
    }
    auto load_a = [&](int kt) {
        const half_t* base = p.A + kt * 64;
        const uint32_t d = (RAGGED && kt == p.KT - 1) ? a_adj : 0u;
#pragma unroll
        for (int it = 0; it < A_LOADS; ++it) areg[it] = *reinterpret_cast<const u32x4_t*>(base + (a_off[it] - d));
    };
    auto store_a = [&](int buf) {
#pragma unroll
        for (int it = 0; it < A_LOADS; ++it) *reinterpret_cast<u32x4_t*>(&As[buf][a_dst[it]]) = areg[it];
    };

    // Packed codes and scale|zero words of the k-tiles in flight: a ring of three slots (tile t in slot t%3, the
    // loads of tile t+2 are issued at the start of tile t, the k-loop is unrolled by three so that slots are
    // compile-time).  With two groups per k-tile the third slot would not fit the register file: current / next
    // (ping-pong with a copy).
    constexpr bool RING = GPT == 1;
    constexpr int NB = RING ? 3 : 2;
    typename WB::Tile bq[NB][FN];
    uint32_t bsz[NB][FN][GPT];
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

    const int a_row0 = (wm * FM * 32 + l32) * kLdsStride + lhi * 8;

    // Pipeline (per wave, MFMAs never stop at a tile boundary):
    //   tile t is computed from LDS buffer t%3 and the codes of its ring slot;
    //   start of tile t : issue the B loads of tile t+2 (ring form; tile t+1 in the ping-pong form): weights come
    //                     from L2/HBM, and a prefetch distance of one tile left part of that latency exposed even
    //                     with two workgroups per CU (measured +1.5 % at 4096 rows, +3 % at 512);
    //   after k-step 0  : park the A registers of tile t+1 (loaded one tile ago) in buffer (t+1)%3, issue
    //                     the A loads of tile t+2, barrier (buffer (t+1)%3 becomes visible; three buffers
    //                     make the write safe against waves still reading tile t-1);
    //   during k-step 3 : the first A fragments of tile t+1 are already read from LDS.
    // Inside a tile the A fragments of the next k-step are read and the next weight fragment is
    // dequantized while the matrix core works on the current one.  On gfx950 an MFMA blocks its own
    // wave's issue for most of its 8 passes, so the dequant VALU mostly overlaps with the MFMAs of the
    // second workgroup resident on the same SIMDs.
    // The loop body is branch-free: loads past the last tile are clamped to the last tile (redundant but
    // harmless, their data is never consumed), so the compiler's wait-count bookkeeping sees one
    // straight-line order of loads and never has to drain the queue conservatively.
    const int last = p.KT - 1;
    load_a(0);
    load_b(0, bq[0], bsz[0]);
    if (RING) load_b(min(1, last), bq[1], bsz[1]);
    store_a(0);
    // Drain the prologue loads here: a load still pending at the loop header would make the compiler
    // place its vmcnt wait inside the loop, where it would also wait for the prefetches just issued.
    __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0)
    load_a(min(1, last));
    __syncthreads();

    half8_t a[2][FM];
#pragma unroll
    for (int fm = 0; fm < FM; ++fm) a[0][fm] = *reinterpret_cast<const half8_t*>(&As[0][a_row0 + fm * 32 * kLdsStride]);
    int buf = 0;
    // one k-tile: weights from slot S, the prefetch (tile kt + DIST) goes to slot P
    auto k_tile = [&](int kt, auto s_c, auto p_c, auto dist_c) {
        constexpr int S = decltype(s_c)::value, P = decltype(p_c)::value, DIST = decltype(dist_c)::value;
        const int nbuf = buf == NBUF - 1 ? 0 : buf + 1;
        load_b(min(kt + DIST, last), bq[P], bsz[P]);
        typename WB::SZ sz[FN][GPT];
#pragma unroll
        for (int fn = 0; fn < FN; ++fn)
#pragma unroll
            for (int g = 0; g < GPT; ++g) sz[fn][g] = WB::expand(bsz[S][fn][g]);
        const half_t* Ab = &As[buf][a_row0];
        const half_t* An = &As[nbuf][a_row0];
        half8_t bcur = WB::dequant(bq[S][0], 0, sz[0][0], magic);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (j == 1) {
                store_a(nbuf);
                load_a(min(kt + 2, last));
                __syncthreads();
            }
#pragma unroll
            for (int fm = 0; fm < FM; ++fm)
                a[(j + 1) & 1][fm] = *reinterpret_cast<const half8_t*>((j + 1 < 4 ? Ab + (j + 1) * 16 : An) + fm * 32 * kLdsStride);
#pragma unroll
            for (int fn = 0; fn < FN; ++fn) {
                const int fnn = fn + 1 < FN ? fn + 1 : 0;
                const int jn = fn + 1 < FN ? j : j + 1;
                half8_t bnext = bcur;
                if (jn < 4) {
                    bnext = WB::dequant(bq[S][fnn], jn, sz[fnn][GPT == 2 ? (jn >> 1) : 0], magic);
                }
#pragma unroll
                for (int fm = 0; fm < FM; ++fm)
                    acc[fm][fn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[j & 1][fm], bcur, acc[fm][fn], 0, 0, 0);
                bcur = bnext;
            }
        }
        buf = nbuf;
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    if constexpr (RING) {
        int kt = 0;
        for (; kt + 3 <= p.KT; kt += 3) {
            k_tile(kt, I0{}, I2{}, I2{});
            k_tile(kt + 1, I1{}, I0{}, I2{});
            k_tile(kt + 2, I2{}, I1{}, I2{});
        }
        if (kt < p.KT) {                           // one or two tiles left, in slots 0 and 1
            k_tile(kt, I0{}, I2{}, I2{});
            if (kt + 1 < p.KT) k_tile(kt + 1, I1{}, I0{}, I2{});
        }
    } else {
        for (int kt = 0; kt < p.KT; ++kt) {
            k_tile(kt, I0{}, I1{}, I1{});
#pragma unroll
            for (int fn = 0; fn < FN; ++fn) {
                bq[0][fn] = bq[1][fn];
#pragma unroll
                for (int g = 0; g < GPT; ++g) bsz[0][fn][g] = bsz[1][fn][g];
            }
        }
    }
    __syncthreads();     // every wave is done with the A tiles: the epilogue reuses the LDS

    // ---- epilogue: transposed through the wave's private LDS region (the A tiles are dead by now) ---
    constexpr int kSlabFloats = 32 * ((EPI == EPI_SWIGLU_F16 ? FN / 2 : FN) * 32 + 8);
    store_tile<EPI, FM, FN>(p, acc, reinterpret_cast<float*>(smem) + wave * kSlabFloats, lane,
                            m0 + wm * FM * 32, (tile_n * WN + wn) * FN, M);
}

// Workgroups the chip holds at once at `occ` per CU (queried once per device).
static int resident_workgroups(int occ) {
    static int cus[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256 * occ;
    if (cus[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cus[dev] = n;
    }
    return cus[dev] * occ;
}

template <int BITS, int WM, int WN, int FM, int FN, int GPT, int EPI, int OCC>
static hipError_t launch_cfg(GemmDev& d, hipStream_t stream) {
    constexpr int BM = WM * FM * 32;
    constexpr int BNF = WN * FN;
    const int rows = (d.tail == 1 && d.rows_exact) ? d.M_max - gemm_tail_rows(d.M_max, d.tail_tiles_n, d.tail_slots) : d.M_max;
    d.tiles_m = (rows + BM - 1) / BM;
    d.tiles_n = (d.vf_total + BNF - 1) / BNF;
    const int blocks = d.tiles_m * d.tiles_n;
    if (blocks == 0) return hipSuccess;
    const dim3 grid(blocks), block(WM * WN * 64);
    if (d.K % 64 != 0)
        hipLaunchKernelGGL((gemm_w4a16_kernel<BITS, WM, WN, FM, FN, GPT, EPI, OCC, true>), grid, block, 0, stream, d);
    else
        hipLaunchKernelGGL((gemm_w4a16_kernel<BITS, WM, WN, FM, FN, GPT, EPI, OCC, false>), grid, block, 0, stream, d);
    return hipGetLastError();
}

template <int BITS, int GPT, int EPI>
static hipError_t launch_epi(GemmDev& d, hipStream_t stream) {
    return launch_cfg<BITS, 1, 4, 4, 2, GPT, EPI, 2>(d, stream);
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

// At most 64 rows (a decode step, or the last rows of a prefill call): one-fragment waves that share activation tiles;
// hidden-size-wide outputs (o-proj, down-proj) also cut K across workgroups when the caller can add the partial tiles.
static hipError_t launch_small_rows(GemmDev& d, const GemmArgs& a, bool parts_ok, hipStream_t stream) {
    const bool resid = a.epilogue == EPI_RESID_F32 || a.epilogue == EPI_RESID_SCATTER;
    // (measured, 7B shape at 64 rows: the 12288-column q|k|v output, whose 192 two-fragment blocks nearly fill the
    // chip without cutting K, takes 17.6 us on the K-sliced skinny kernel and 20.3 us on the decode kernel)
    const bool wide_store = a.epilogue == EPI_STORE_F16 && d.M_max > 32 && d.vf_total >= 256;
    if (!resid && !wide_store) {
        int nwn;
        gemm_decode_plan(d, a.epilogue, 1, &nwn);
        return launch_gemm_decode(d, a.epilogue, nwn, 1, stream);
    }
    if (parts_ok && a.part && a.n_parts) {
        int nwn;
        const int split = gemm_decode_plan(d, EPI_PARTIAL_F32, kGemmPartMax, &nwn);
        d.out = a.part;
        *a.n_parts = split;
        return launch_gemm_decode(d, EPI_PARTIAL_F32, nwn, split, stream);
    }
    return launch_gemm_skinny(d, a.epilogue, stream);
}

hipError_t launch_gemm_w4a16(const GemmArgs& a, hipStream_t stream) {
    if (a.M_max <= 0) return hipSuccess;
    GemmDev d{};
    d.A = reinterpret_cast<const half_t*>(a.A);
    d.count = a.count;
    d.M_max = a.M_max;
    d.rows_exact = a.rows_exact;
    d.K = a.K;
    d.KT = (a.K + 63) / 64;
    d.gshift = a.group == 32 ? 5 : a.group == 64 ? 6 : 7;
    d.n_w = a.n_w;
    int col = 0, vf = 0;
    for (int i = 0; i < 3; ++i) {
        const int j = i < a.n_w ? i : 0;
        const PrepackDims pd = prepack_dims(a.w[j].N, a.w[j].K, a.group, a.bits);
        d.codes[i] = a.w[j].prepacked;
        d.sz[i] = reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(a.w[j].prepacked) + pd.code_bytes);
        d.N[i] = a.w[j].N;
        d.NF[i] = pd.NF;
        d.npad[i] = pd.NF * 32;
        d.colbase[i] = col;
        if (i < a.n_w) { col += a.w[j].N; vf += pd.NF; }
    }
    d.vf_total = vf;
    d.out = a.out;
    d.ldo = a.ldo;
    d.resid = a.resid;
    d.idx = a.idx;
    d.bf16 = a.bf16;
    d.bits = a.bits;
    // Few rows: the weight stream dominates and 128-row tiles cannot fill the chip (a 5120-column output is 20
    // workgroups).  Up to 64 rows the skinny kernel streams the weights once; up to 256 rows it runs one 64-row
    // chunk per workgroup (measured on 13B-shaped linears at 128 rows: 26-59 us against 64-178 us here; at 256
    // rows the two are level).
    if (a.n_parts) *a.n_parts = 0;
    if (d.M_max <= kGemmPartRows) return launch_small_rows(d, a, true, stream);
    if (d.M_max <= 256) return launch_gemm_skinny(d, a.epilogue, stream);
    // A few hundred rows: so few 128 x 256 tiles that a CU holds at most one workgroup, whose k-loop then runs
    // at one memory latency per k-tile.  The 64-row kernel with its deep prefetch rings takes over while its own
    // grid fits the chip in one round (measured crossovers on 7B- and 13B-shaped linears: 2.5 workgroups per CU
    // for the one-fragment form, 2 per CU for the gate/up form).
    {
        const bool swiglu = a.epilogue == EPI_SWIGLU_F16;
        const int mid_tiles = ((d.M_max + 63) / 64) * ((d.vf_total + (swiglu ? 7 : 3)) / (swiglu ? 8 : 4));
        const int cus = resident_workgroups(1);
        if (swiglu ? mid_tiles <= 2 * cus : 2 * mid_tiles <= 5 * cus) return launch_gemm_mid(d, a.epilogue, stream);
    }
    // 128-row tiles from here on; the rows after the last full tile may go to the small-row kernels (gemm_tail_rows).
    // With a device-side count (threshold mode) the tail launch is always made and decides on the device.
    if (d.M_max >= 128) {
        d.tail_tiles_n = (d.vf_total + 7) / 8;              // launch_epi: 4 waves x 2 fragments per workgroup
        d.tail_slots = resident_workgroups(2);
        const int tail_bound = a.rows_exact ? gemm_tail_rows(d.M_max, d.tail_tiles_n, d.tail_slots) : 127;
        if (tail_bound > 0) {
            GemmDev t = d;
            t.tail = 2; t.M_full = d.M_max; t.M_max = tail_bound;
            const hipError_t e = tail_bound <= kGemmPartRows ? launch_small_rows(t, a, false, stream)
                                                             : launch_gemm_skinny(t, a.epilogue, stream);
            if (e != hipSuccess) return e;
            d.tail = 1;
        }
    }
    if (a.bits == 3) {
        if (a.group == 32) return launch_gpt<3, 2>(d, a.epilogue, stream);
        return launch_gpt<3, 1>(d, a.epilogue, stream);
    }
    if (a.bits == 2) {
        if (a.group == 32) return launch_gpt<2, 2>(d, a.epilogue, stream);
        return launch_gpt<2, 1>(d, a.epilogue, stream);
    }
    if (a.group == 32) return launch_gpt<4, 2>(d, a.epilogue, stream);
    return launch_gpt<4, 1>(d, a.epilogue, stream);
}

}  // namespace qtale
