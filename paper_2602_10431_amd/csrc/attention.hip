// Attention restricted to executed tokens.
//
// A bypassed token produces no query, key or value at a layer (the whole layer is skipped for it, Eq. 3),
// so an executed token attends causally to the executed tokens of its own sequence only, in original
// order, preceded by that layer's cache entries (which also hold executed tokens only).  Rows of the
// compact q|k|v buffer are in ascending token order, so the executed tokens of sequence b are the rows
// cu_exec[b] .. cu_exec[b+1]-1 and "causal" means "row index <= own row index".
//
// Two kernels:
//   * flash_prefill: matrix-core tiles.  A workgroup of 4 waves owns 128 query rows of one (sequence,
//     head); keys/values stream through LDS in tiles of 64.  S^T = K Q^T is computed so that a lane owns
//     one query column (softmax statistics are per lane), and the probabilities, still in the MFMA
//     accumulator layout, are fed straight back as the B operand of O^T = V^T P^T; V is transposed on
//     its way into LDS.
//   * decode: one workgroup per (executed row, kv head); lanes stream K and V rows with 16-byte loads,
//     16 (or 8) lanes per key, online softmax per lane group, merged at the end.  Bandwidth-bound.
#include <algorithm>
#include <type_traits>

#include "qtale_dev.h"
#include "qtale_kernels.h"

namespace qtale {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;

struct AttnDev {
    const half_t* qkv;
    half_t* out;
    int nh, nkv, width;          // width = (nh + 2 nkv) * d
    const int32_t* count;
    const int32_t* cu_exec;
    const int32_t* row_seq;
    const int4* items;           // prefill work list: (sequence or -1, query tile, first compact row, rows) per item
    const int32_t* n_items;
    int items_max;               // host bound on the number of work items (row stride of the logical grid)
    const half_t* k_cache;
    const half_t* v_cache;
    const int32_t* kv_old;
    int cap;
    float scale_log2;            // log2(e) / sqrt(d)
    float* part;                 // decode, split keys: [row][head][split][D + 2] fp32 (numerators, maximum, denominator)
    int n_split;                 // key ranges per (row, kv head); 1 = no split
};

template <int D>
__global__ void __launch_bounds__(256, 2)
flash_prefill_kernel(AttnDev p) {
    constexpr int KS = D / 16;          // k-steps of the QK^T product
    constexpr int DF = D / 32;          // 32-wide fragments of the head dimension
    constexpr int KSTR = D + 8;         // LDS row stride of the K tile (halves)
    // Transposed V tile Vt[column][key]: 64 keys + room for the column skew, row stride 42 dwords (16 lanes that read
    // 8 bytes of consecutive rows hit 16 different bank pairs).  A thread stores 4 keys (8 bytes) of 8 columns; the
    // 16 lanes that hold the same keys and 16 different column chunks dc would land on two bank pairs, so the key
    // group index is XOR-ed with dc >> 2 (uniform per 32-column fragment on the read side) and rows with bit 1 of dc
    // set are shifted by 8 dwords: bits 1-2, 3 and 4 of the bank index then come from dc >> 2, dc bit 1 and dc bit 0.
    constexpr int VSTR = 64 + 16 + 4;   // LDS row stride of the transposed V tile (halves)
    constexpr int CPR = D / 8;          // 16-byte chunks per K/V row
    constexpr int CH = (64 * CPR) / 256;     // K chunks per thread per tile
    constexpr int VG = (16 * CPR + 255) / 256;   // V groups (4 keys x 8 columns) per thread per tile
    constexpr int kSwShift = CPR == 8 ? 1 : 0;   // 8 chunks per row: two key groups share 16 lanes, swizzle bit 1 instead of bit 0
    __shared__ __attribute__((aligned(16))) half_t Ks2[2][64 * KSTR];    // double-buffered tiles
    __shared__ __attribute__((aligned(16))) half_t Vt2[2][D * VSTR];

    // Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  Every XCD gets a contiguous group of
    // heads (all query heads of a few key/value heads) and walks the work items in list order, the heads of the group
    // innermost: the list is sorted by length, longest first, so an XCD's 64 workgroup slots drain evenly (with the
    // heads outermost the long items of the last head started when most of the work was done: about a third of the
    // kernel time at two sequences of 4096 tokens was an idle tail), and the workgroups that run at the same time
    // belong to a few (sequence, head) pairs and similar key ranges, which the L2 serves.
    int h, item;
    if ((p.nh & 7) == 0) {
        const int hx = p.nh >> 3;                                // heads per XCD; gridDim.x = 8 * hx * items_max
        const int local = blockIdx.x >> 3;
        item = local / hx;
        h = (blockIdx.x & 7) * hx + (local - item * hx);
    } else {
        const int per_xcd = gridDim.x >> 3;
        const int L = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
        h = L / p.items_max;
        item = L - h * p.items_max;
    }
    if (h >= p.nh) return;
    const int4 it = p.items[item];           // one load tells the workgroup everything (unused slots hold -1)
    const int b = it.x, qt = it.y;
    if (b < 0) return;
    const int hk = h / (p.nh / p.nkv);
    const int row_begin = it.z;
    const int n_b = it.w;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lhi = lane >> 5;

    // key/value source: the layer cache (new rows were appended before this kernel) or the compact buffer
    const half_t* kbase;
    const half_t* vbase;
    int kv_stride, base_len;
    if (p.k_cache) {
        base_len = p.kv_old[b];
        kv_stride = D;                                           // cache [B][n_kv_heads][cap][D]: a head's entries are contiguous
        kbase = p.k_cache + (static_cast<size_t>(b) * p.nkv + hk) * p.cap * D;
        vbase = p.v_cache + (static_cast<size_t>(b) * p.nkv + hk) * p.cap * D;
    } else {
        base_len = 0;
        kv_stride = p.width;
        kbase = p.qkv + static_cast<size_t>(row_begin) * p.width + (p.nh + hk) * D;
        vbase = kbase + p.nkv * D;
    }
    const int q_lo = qt * kAttnBQ;                               // first local query index of the block
    const int q_cnt = min(kAttnBQ, n_b - q_lo);
    int n_keys = base_len + q_lo + q_cnt;                        // keys visible to the last query
    if (p.k_cache) n_keys = min(n_keys, p.cap);
    const int n_tiles = (n_keys + 63) / 64;

    // this lane's query (column of S^T): local index inside the sequence, clamped to a valid row
    const int q_local = q_lo + min(wave * 32 + l32, q_cnt - 1);
    const int limit = base_len + q_local + 1;                    // keys [0, limit) are visible
    const int wave_hi = base_len + q_lo + min(wave * 32 + 31, q_cnt - 1) + 1;   // largest limit in the wave
    const int wave_lo = base_len + q_lo + min(wave * 32, q_cnt - 1) + 1;        // smallest limit in the wave
    const half_t* qrow = p.qkv + static_cast<size_t>(row_begin + q_local) * p.width + h * D;
    // The queries stay as stored; the factor log2(e)/sqrt(d) is applied in fp32 inside the exponent's fused
    // multiply-add (folding it into the fp16 queries would round it, and every product, to 11 bits: an error in
    // the logits that grows with their magnitude).
    half8_t qf[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = *reinterpret_cast<const half8_t*>(qrow + 16 * s + 8 * lhi);
    const float sc = p.scale_log2;

    float16_t o[DF];
#pragma unroll
    for (int df = 0; df < DF; ++df)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[df][r] = 0.0f;
    float m_run = kNegBig, l_run = 0.0f;

    // global -> register staging of one tile.  K: chunk c is key c / CPR, 8 halves at (c % CPR)*8.
    // V: a thread owns 4 consecutive keys x 8 columns and transposes them in registers, so that the
    // transposed tile Vt[column][key] is written with 8-byte stores.
    // One register set: tile t+1 waits in it while tile t is computed.
    // Element offsets inside a tile are fixed per thread; a tile adds key0 * kv_stride, and the minimum with the
    // offset of the same column chunk in the last visible key keeps the (partial) last tile inside the sequence.
    u32x4_t kregs[CH], vregs[VG][4];
    uint32_t k_off[CH], k_max[CH], v_off[VG], v_max[VG];            // byte offsets (below 4 GB: 32-bit lane offsets on a uniform base)
    const uint32_t row_bytes = static_cast<uint32_t>(kv_stride) * 2u;
    const uint32_t last_row = static_cast<uint32_t>(n_keys - 1) * row_bytes;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int c = i * 256 + tid;
        k_off[i] = static_cast<uint32_t>(c / CPR) * row_bytes + (c % CPR) * 16;
        k_max[i] = last_row + (c % CPR) * 16;
    }
#pragma unroll
    for (int i = 0; i < VG; ++i) {
        const int g = min(i * 256 + tid, 16 * CPR - 1);
        v_off[i] = static_cast<uint32_t>(4 * (g / CPR)) * row_bytes + (g % CPR) * 16;
        v_max[i] = last_row + (g % CPR) * 16;
    }
    const char* kbytes = reinterpret_cast<const char*>(kbase);
    const char* vbytes = reinterpret_cast<const char*>(vbase);
    auto fetch = [&](int tile, u32x4_t* kreg, u32x4_t (*vreg)[4]) {
        const uint32_t t_off = static_cast<uint32_t>(tile * 64) * row_bytes;
#pragma unroll
        for (int i = 0; i < CH; ++i)
            kreg[i] = *reinterpret_cast<const u32x4_t*>(kbytes + min(k_off[i] + t_off, k_max[i]));
#pragma unroll
        for (int i = 0; i < VG; ++i)
#pragma unroll
            for (int u = 0; u < 4; ++u)
                vreg[i][u] = *reinterpret_cast<const u32x4_t*>(vbytes + min(v_off[i] + t_off + static_cast<uint32_t>(u) * row_bytes, v_max[i]));
    };
    auto stage = [&](int buf, const u32x4_t* kreg, const u32x4_t (*vreg)[4]) {
        half_t* Ks = Ks2[buf];
        half_t* Vt = Vt2[buf];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = i * 256 + tid;
            *reinterpret_cast<u32x4_t*>(&Ks[(c / CPR) * KSTR + (c % CPR) * 8]) = kreg[i];
        }
#pragma unroll
        for (int i = 0; i < VG; ++i) {
            const int g = i * 256 + tid;
            if (g >= 16 * CPR) continue;
            const int kg = g / CPR, dc = g % CPR;
            const int vcol = 4 * (kg ^ ((dc >> 2) << kSwShift)) + 16 * ((dc >> 1) & 1);
#pragma unroll
            for (int w = 0; w < 4; ++w) {                        // word w holds columns 2w, 2w+1 of each key
                const uint32_t a0 = vreg[i][0][w], a1 = vreg[i][1][w], a2 = vreg[i][2][w], a3 = vreg[i][3][w];
                uint2 even, odd;
                even.x = (a0 & 0xffffu) | (a1 << 16);
                even.y = (a2 & 0xffffu) | (a3 << 16);
                odd.x = (a0 >> 16) | (a1 & 0xffff0000u);
                odd.y = (a2 >> 16) | (a3 & 0xffff0000u);
                *reinterpret_cast<uint2*>(&Vt[(dc * 8 + 2 * w) * VSTR + vcol]) = even;
                *reinterpret_cast<uint2*>(&Vt[(dc * 8 + 2 * w + 1) * VSTR + vcol]) = odd;
            }
        }
    };

    // Tile t+1 is parked in the other LDS buffer and tile t+2 requested before tile t is computed: one barrier per
    // tile, a whole tile time to cover the latency of a fetch, and the staging of one wave overlaps the MFMAs of the
    // others.
    fetch(0, kregs, vregs);
    stage(0, kregs, vregs);
    if (n_tiles > 1) fetch(1, kregs, vregs);
    __syncthreads();
    // this lane's row of a V^T fragment: row l32, shifted by the row's skew; key group lhi (v_rd0) or 1 - lhi (v_rd1:
    // fragments whose swizzle flips bit 0 of the key group)
    const int v_row = l32 * VSTR + 16 * ((l32 >> 4) & 1);
    const int v_rd0 = v_row + 4 * lhi, v_rd1 = v_row + 4 * (1 - lhi);
    for (int tile = 0; tile < n_tiles; ++tile) {
        if (tile + 1 < n_tiles) stage((tile + 1) & 1, kregs, vregs);
        if (tile + 2 < n_tiles) fetch(tile + 2, kregs, vregs);
        const half_t* Ks = Ks2[tile & 1];
        const half_t* Vt = Vt2[tile & 1];
        const int key0 = tile * 64;
        if (key0 < wave_hi) {
            // S^T = K Q^T : rows = keys (two 32-key fragments), column = this lane's query
            // (the fragments of the whole tile are named before the MFMAs so that the compiler may issue their reads as
            // early as registers allow)
            float16_t st[2];
            half8_t ka[2][KS];
#pragma unroll
            for (int kf = 0; kf < 2; ++kf)
#pragma unroll
                for (int s = 0; s < KS; ++s)
                    ka[kf][s] = *reinterpret_cast<const half8_t*>(&Ks[(kf * 32 + l32) * KSTR + 16 * s + 8 * lhi]);
#pragma unroll
            for (int kf = 0; kf < 2; ++kf) {
#pragma unroll
                for (int r = 0; r < 16; ++r) st[kf][r] = 0.0f;
#pragma unroll
                for (int s = 0; s < KS; ++s) st[kf] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ka[kf][s], qf[s], st[kf], 0, 0, 0);
            }
            // online softmax over the 32 scores this lane holds (the lane 32 away holds the other 32);
            // only tiles that reach past the wave's smallest causal limit need the mask
            if (key0 + 64 > wave_lo) {
#pragma unroll
                for (int kf = 0; kf < 2; ++kf)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = key0 + kf * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3);
                        if (key >= limit) st[kf][r] = kNegBig;
                    }
            }
            float mx = kNegBig;
#pragma unroll
            for (int kf = 0; kf < 2; ++kf)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, st[kf][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            // Reference point of the exponentials, in units of log2 (sc > 0: same arg-max).  Any value works as long
            // as numerators and denominator share it, so it only follows the running maximum when some lane's maximum
            // has grown by more than kLazy (probabilities then stay below 2^kLazy, far inside fp16): with 64 queries
            // per wave some maximum moves in most tiles, and rescaling the 64 output accumulators every time costs a
            // fifth of the kernel's vector instructions.
            constexpr float kLazy = 4.0f;
            const float m_cand = fmaxf(m_run, mx * sc);
            const float m_new = __any(m_cand > m_run + kLazy) ? m_cand : m_run;
            float psum = 0.0f;
            half8_t pf[4];
#pragma unroll
            for (int kf = 0; kf < 2; ++kf)
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    float2_t pv;
                    pv[0] = __builtin_amdgcn_exp2f(fmaf(st[kf][r], sc, -m_new));
                    pv[1] = __builtin_amdgcn_exp2f(fmaf(st[kf][r + 1], sc, -m_new));
                    psum += pv[0] + pv[1];
                    const half2_t ph = __builtin_convertvector(pv, half2_t);   // one packed conversion per pair
                    pf[kf * 2 + (r >> 3)][r & 7] = ph[0];
                    pf[kf * 2 + (r >> 3)][(r & 7) + 1] = ph[1];
                }
            if (__any(m_new != m_run)) {                         // rescale only when the reference point moved
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
                l_run *= alpha;
#pragma unroll
                for (int df = 0; df < DF; ++df)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[df][r] *= alpha;
                m_run = m_new;
            }
            l_run += psum;
            // O^T += V^T P^T : k-step s2 covers keys 16 s2 .. 16 s2 + 15 of the tile; operand element e of a
            // lane is key 16 s2 + 8 (e/4) + 4 (lane/32) + e%4, the order the accumulator layout produced
            half8_t va[4][DF];
#pragma unroll
            for (int s2 = 0; s2 < 4; ++s2) {
#pragma unroll
                for (int df = 0; df < DF; ++df) {
                    // key groups 4 s2 + lhi and 4 s2 + 2 + lhi of column df * 32 + l32, at their swizzled places
                    const int sw = df << kSwShift;               // (dc >> 2) << kSwShift with dc = (df * 32 + l32) >> 3
                    const half_t* vrow = &Vt[(df * 32) * VSTR] + ((sw & 1) ? v_rd1 : v_rd0);
                    const half4_t v0 = *reinterpret_cast<const half4_t*>(vrow + 4 * ((4 * s2) ^ (sw & ~1)));
                    const half4_t v1 = *reinterpret_cast<const half4_t*>(vrow + 4 * ((4 * s2 + 2) ^ (sw & ~1)));
                    va[s2][df][0] = v0[0]; va[s2][df][1] = v0[1]; va[s2][df][2] = v0[2]; va[s2][df][3] = v0[3];
                    va[s2][df][4] = v1[0]; va[s2][df][5] = v1[1]; va[s2][df][6] = v1[2]; va[s2][df][7] = v1[3];
                }
            }
#pragma unroll
            for (int s2 = 0; s2 < 4; ++s2)
#pragma unroll
                for (int df = 0; df < DF; ++df) o[df] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va[s2][df], pf[s2], o[df], 0, 0, 0);
        }
        __syncthreads();
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_tot;
    if (wave * 32 + l32 < q_cnt) {
        half_t* orow = p.out + static_cast<size_t>(row_begin + q_local) * (p.nh * D) + h * D;
#pragma unroll
        for (int df = 0; df < DF; ++df)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                half4_t v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = static_cast<half_t>(o[df][4 * g + e] * inv);
                *reinterpret_cast<half4_t*>(orow + df * 32 + 8 * g + 4 * lhi) = v;
            }
    }
}

// Builds the prefill work list: one item per (sequence, tile of kAttnBQ executed rows), carrying the sequence's
// first compact row and row count so that the attention workgroups need no further lookups; the slots up to
// items_max that no tile uses are marked with sequence -1.  The list is sorted by query tile index, highest
// first, across all sequences (the tile index is the item's length in keys up to the cached prefix): a counting
// sort over the tiles-per-sequence histogram.  `levels` is the host bound on tiles per sequence (<= kItemLevels).
constexpr int kItemLevels = 1024;

__global__ void __launch_bounds__(256)
attn_items_kernel(const int32_t* __restrict__ cu_exec, int B, int4* __restrict__ items, int items_max,
                  int32_t* __restrict__ n_items, int levels) {
    __shared__ int cnt[kItemLevels + 1];      // first: sequences with exactly n tiles; then: sequences with more than n
    __shared__ int offs[kItemLevels + 1];     // items of the tile indices above q
    __shared__ int fill[kItemLevels + 1];
    __shared__ int s_total;
    const int tid = threadIdx.x, lane = tid & 63;
    for (int i = tid; i <= levels; i += 256) { cnt[i] = 0; fill[i] = 0; }
    __syncthreads();
    for (int b = tid; b < B; b += 256) {
        const int nt = min((cu_exec[b + 1] - cu_exec[b] + kAttnBQ - 1) / kAttnBQ, levels);
        atomicAdd(&cnt[nt], 1);
    }
    __syncthreads();
    if (tid < 64) {
        // two suffix sums over the levels, one wave: lane l owns a chunk of consecutive levels
        const int chunk = (levels + 64) / 64;
        const int lo = lane * chunk, hi = min(lo + chunk, levels + 1);
        int own = 0;
        for (int n = lo; n < hi; ++n) own += cnt[n];
        int above = 0;                                           // sum of the chunks of the lanes above
        {
            int incl = own;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_down(incl, o, 64);
                if (lane + o < 64) incl += t;
            }
            above = incl - own;
        }
        int own2 = 0;
        for (int n = hi - 1; n >= lo; --n) {
            const int h = cnt[n];
            cnt[n] = above;                                      // sequences with more than n tiles
            own2 += above;
            above += h;
        }
        int above2 = 0;
        {
            int incl = own2;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_down(incl, o, 64);
                if (lane + o < 64) incl += t;
            }
            above2 = incl - own2;
        }
        for (int n = hi - 1; n >= lo; --n) {
            offs[n] = above2;                                    // items with a tile index above n
            above2 += cnt[n];
        }
        if (lane == 0) s_total = above2;                         // lane 0 ends below level 0: all items
    }
    __syncthreads();
    for (int b = tid; b < B; b += 256) {
        const int first = cu_exec[b];
        const int rows = cu_exec[b + 1] - first;
        const int nt = min((rows + kAttnBQ - 1) / kAttnBQ, levels);
        if (nt == 0) continue;
        const int pos = cnt[nt] + atomicAdd(&fill[nt], 1);        // place among the sequences, most tiles first
        for (int q = 0; q < nt; ++q) items[offs[q] + pos] = make_int4(b, q, first, rows);
    }
    const int used = s_total;
    for (int i = used + tid; i < items_max; i += 256) items[i] = make_int4(-1, 0, 0, 0);
    if (tid == 0) *n_items = used;
}

// The same list for calls whose sequences could have more than kItemLevels query tiles: sequence by sequence, each
// sequence's tiles longest first.
__global__ void __launch_bounds__(256)
attn_items_by_sequence_kernel(const int32_t* __restrict__ cu_exec, int B, int4* __restrict__ items, int items_max,
                              int32_t* __restrict__ n_items) {
    __shared__ int s_wave[4];
    __shared__ int s_base;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) s_base = 0;
    __syncthreads();
    for (int b0 = 0; b0 < B; b0 += 256) {
        const int b = b0 + threadIdx.x;
        const int first = b < B ? cu_exec[b] : 0;
        const int rows = b < B ? cu_exec[b + 1] - first : 0;
        const int nt = (rows + kAttnBQ - 1) / kAttnBQ;
        int incl = nt;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o, 64);
            if (lane >= o) incl += t;
        }
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        int start = s_base + incl - nt;
        for (int w = 0; w < wave; ++w) start += s_wave[w];
        for (int q = 0; q < nt; ++q) items[start + q] = make_int4(b, nt - 1 - q, first, rows);   // longest tiles first
        __syncthreads();
        if (threadIdx.x == 0) s_base += s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
        __syncthreads();
    }
    const int used = s_base;
    for (int i = used + threadIdx.x; i < items_max; i += 256) items[i] = make_int4(-1, 0, 0, 0);
    if (threadIdx.x == 0) *n_items = used;
}

// Sum over the LPK (8 or 16) adjacent lanes that share a key, left in every one of them.  Data-parallel-primitive
// modifiers on the adds (quad permutes, then mirror within 8 and within 16 lanes: after the quad steps the
// lanes of a quad hold equal values, so a mirror exchanges whole quads / halves) instead of cross-lane moves
// through the LDS crossbar: the dot products of a decode step need 4 such sums per key and query head.
template <int LPK>
__device__ __forceinline__ float key_group_sum(float x) {
    static_assert(LPK == 8 || LPK == 16, "8 or 16 lanes per key");
    auto step = [](float v, auto ctrl) {
        const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), decltype(ctrl)::value, 0xf, 0xf, true);
        return v + __builtin_bit_cast(float, moved);
    };
    x = step(x, std::integral_constant<int, 0xB1>{});       // quad_perm [1,0,3,2]
    x = step(x, std::integral_constant<int, 0x4E>{});       // quad_perm [2,3,0,1]
    x = step(x, std::integral_constant<int, 0x141>{});      // row_half_mirror
    if (LPK == 16) x = step(x, std::integral_constant<int, 0x140>{});   // row_mirror
    return x;
}

// Decode-style attention: workgroup = (executed row, kv head); REP query heads share the kv head.
// SPLIT: with few rows there are fewer workgroups than the chip needs to saturate HBM (8 rows x 32 kv heads is
// one workgroup per CU: 4.1 TB/s against 6.0 with eight per CU), so the keys of a (row, kv head) are cut into
// n_split contiguous ranges (multiples of the 64- or 128-key step) that separate workgroups stream; each writes
// its unnormalised sums with their maximum and denominator, and attn_merge_kernel combines the ranges in order.
template <int D, int REP, bool SPLIT>
__global__ void __launch_bounds__(256)
attn_decode_kernel(AttnDev p) {
    constexpr int LPK = D / 8;            // lanes per key (each lane owns 8 of the D columns)
    constexpr int KPW = 64 / LPK;         // keys per wave per step
    constexpr int UNR = 4;
    // kv head fastest: the workgroups of one executed row are launched together
    const int i = blockIdx.y;
    if (i >= *p.count) return;
    const int hk = blockIdx.x;
    const int b = p.row_seq[i];
    const int row_begin = p.cu_exec[b];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane % LPK, slot = lane / LPK;

    const half_t* kbase;
    const half_t* vbase;
    int kv_stride, n_keys;
    if (p.k_cache) {
        kv_stride = D;                        // cache [B][n_kv_heads][cap][D]: one contiguous stream per workgroup
        kbase = p.k_cache + (static_cast<size_t>(b) * p.nkv + hk) * p.cap * D;
        vbase = p.v_cache + (static_cast<size_t>(b) * p.nkv + hk) * p.cap * D;
        n_keys = min(p.kv_old[b] + (i - row_begin) + 1, p.cap);
    } else {
        kv_stride = p.width;
        kbase = p.qkv + static_cast<size_t>(row_begin) * p.width + (p.nh + hk) * D;
        vbase = kbase + p.nkv * D;
        n_keys = i - row_begin + 1;
    }

    float q[REP][8];
#pragma unroll
    for (int r = 0; r < REP; ++r) {
        const half8_t qv = *reinterpret_cast<const half8_t*>(p.qkv + static_cast<size_t>(i) * p.width + (hk * REP + r) * D + sub * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) q[r][e] = static_cast<float>(qv[e]) * p.scale_log2;
    }
    float m_run[REP], l_run[REP], o[REP][8];
#pragma unroll
    for (int r = 0; r < REP; ++r) {
        m_run[r] = kNegBig;
        l_run[r] = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[r][e] = 0.0f;
    }

    const int step = 4 * KPW;             // keys per workgroup step
    int key_lo = 0, key_hi = n_keys;      // this workgroup's key range
    if (SPLIT) {
        const int gran = UNR * step;
        const int per = ((n_keys + p.n_split - 1) / p.n_split + gran - 1) / gran * gran;
        key_lo = min(static_cast<int>(blockIdx.z) * per, n_keys);
        key_hi = min(key_lo + per, n_keys);
    }
    // The keys and values of the next step are requested before the current step is consumed, so the memory
    // pipe never drains while the lanes do their dot products and exponentials (keys past the end are clamped
    // to the last one and masked).
    half8_t kn[UNR], vn[UNR];
    auto fetch = [&](int kb) {
        const int k0 = kb + wave * KPW + slot;
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int kc = min(k0 + u * step, n_keys - 1);      // n_keys >= 1: always a valid row
            kn[u] = *reinterpret_cast<const half8_t*>(kbase + static_cast<size_t>(kc) * kv_stride + sub * 8);
            vn[u] = *reinterpret_cast<const half8_t*>(vbase + static_cast<size_t>(kc) * kv_stride + sub * 8);
        }
    };
    fetch(key_lo);
    for (int kb = key_lo; kb < key_hi; kb += UNR * step) {     // trip count is uniform over the workgroup
        const int k0 = kb + wave * KPW + slot;
        half8_t kv[UNR], vv[UNR];
        bool ok[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            ok[u] = k0 + u * step < key_hi;
            kv[u] = kn[u];
            vv[u] = vn[u];
        }
        fetch(min(kb + UNR * step, n_keys - 1));               // past the end: one redundant, unused fetch
#pragma unroll
        for (int r = 0; r < REP; ++r) {
            float s[UNR];
            float mx = m_run[r];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                float acc = 0.0f;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc = fmaf(q[r][e], static_cast<float>(kv[u][e]), acc);
                acc = key_group_sum<LPK>(acc);
                s[u] = ok[u] ? acc : kNegBig;
                mx = fmaxf(mx, s[u]);
            }
            const float alpha = exp2f(m_run[r] - mx);
            m_run[r] = mx;
            float lsum = l_run[r] * alpha;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[r][e] *= alpha;
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const float pv = ok[u] ? exp2f(s[u] - mx) : 0.0f;
                lsum += pv;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[r][e] = fmaf(pv, static_cast<float>(vv[u][e]), o[r][e]);
            }
            l_run[r] = lsum;
        }
    }

    // merge the key slots of a wave (lanes that own the same columns), then the four waves through LDS
    __shared__ float sm[4][REP][D + 2];
#pragma unroll
    for (int r = 0; r < REP; ++r) {
#pragma unroll
        for (int off = LPK; off < 64; off <<= 1) {
            const float m2 = __shfl_xor(m_run[r], off, 64);
            const float l2 = __shfl_xor(l_run[r], off, 64);
            const float mn = fmaxf(m_run[r], m2);
            const float a1 = exp2f(m_run[r] - mn), a2 = exp2f(m2 - mn);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float o2 = __shfl_xor(o[r][e], off, 64);
                o[r][e] = o[r][e] * a1 + o2 * a2;
            }
            l_run[r] = l_run[r] * a1 + l2 * a2;
            m_run[r] = mn;
        }
        if (slot == 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) sm[wave][r][sub * 8 + e] = o[r][e];
            if (sub == 0) { sm[wave][r][D] = m_run[r]; sm[wave][r][D + 1] = l_run[r]; }
        }
    }
    __syncthreads();
    for (int c = tid; c < REP * D; c += 256) {
        const int r = c / D, e = c % D;
        float mn = kNegBig;
#pragma unroll
        for (int w = 0; w < 4; ++w) mn = fmaxf(mn, sm[w][r][D]);
        float num = 0.0f, den = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float a = exp2f(sm[w][r][D] - mn);
            num += sm[w][r][e] * a;
            den += sm[w][r][D + 1] * a;
        }
        if (SPLIT) {
            // an empty range leaves num = 0, den = 0 and the maximum at its initial value: it drops out of the merge
            float* dst = p.part + ((static_cast<size_t>(i) * p.nh + hk * REP + r) * p.n_split + blockIdx.z) * (D + 2);
            dst[e] = num;
            if (e == 0) { dst[D] = mn; dst[D + 1] = den; }
        } else {
            p.out[static_cast<size_t>(i) * (p.nh * D) + (hk * REP + r) * D + e] = static_cast<half_t>(num / den);
        }
    }
}

// Combines the key ranges of the split decode kernel: out = sum_s num_s 2^(m_s - m) / sum_s den_s 2^(m_s - m),
// ranges taken in order.  One workgroup per (row, 256 / D heads).
template <int D>
__global__ void __launch_bounds__(256)
attn_merge_kernel(AttnDev p) {
    const int i = blockIdx.y;
    if (i >= *p.count) return;
    const int head = blockIdx.x * (256 / D) + threadIdx.x / D;
    const int e = threadIdx.x % D;
    if (head >= p.nh) return;
    const float* src = p.part + (static_cast<size_t>(i) * p.nh + head) * p.n_split * (D + 2);
    float mn = kNegBig;
    for (int s = 0; s < p.n_split; ++s) mn = fmaxf(mn, src[s * (D + 2) + D]);
    float num = 0.0f, den = 0.0f;
    for (int s = 0; s < p.n_split; ++s) {
        const float a = exp2f(src[s * (D + 2) + D] - mn);
        num += src[s * (D + 2) + e] * a;
        den += src[s * (D + 2) + D + 1] * a;
    }
    p.out[static_cast<size_t>(i) * (p.nh * D) + head * D + e] = static_cast<half_t>(num / den);
}

// CUs of the current device (queried once per device).
static int attn_cus() {
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

template <int D, bool SPLIT>
static hipError_t launch_decode_rep(const AttnDev& d, int rep, int rows, int nkv, hipStream_t stream) {
    const dim3 grid(nkv, rows, SPLIT ? d.n_split : 1), block(256);
    switch (rep) {
        case 1: hipLaunchKernelGGL((attn_decode_kernel<D, 1, SPLIT>), grid, block, 0, stream, d); break;
        case 2: hipLaunchKernelGGL((attn_decode_kernel<D, 2, SPLIT>), grid, block, 0, stream, d); break;
        case 4: hipLaunchKernelGGL((attn_decode_kernel<D, 4, SPLIT>), grid, block, 0, stream, d); break;
        case 8: hipLaunchKernelGGL((attn_decode_kernel<D, 8, SPLIT>), grid, block, 0, stream, d); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int D>
static hipError_t launch_decode_d(const AttnDev& d, int rep, int rows, int nkv, hipStream_t stream) {
    if (d.n_split <= 1) return launch_decode_rep<D, false>(d, rep, rows, nkv, stream);
    hipError_t e = launch_decode_rep<D, true>(d, rep, rows, nkv, stream);
    if (e != hipSuccess) return e;
    const dim3 grid((d.nh * D + 255) / 256, rows), block(256);
    hipLaunchKernelGGL(attn_merge_kernel<D>, grid, block, 0, stream, d);
    return hipGetLastError();
}

hipError_t launch_attention(const AttnArgs& a, hipStream_t stream) {
    if (a.max_rows == 0) return hipSuccess;
    AttnDev d{};
    d.qkv = reinterpret_cast<const half_t*>(a.qkv);
    d.out = reinterpret_cast<half_t*>(a.out);
    d.nh = a.nh;
    d.nkv = a.nkv;
    d.width = (a.nh + 2 * a.nkv) * a.d;
    d.count = a.count;
    d.cu_exec = a.cu_exec;
    d.row_seq = a.row_seq;
    d.items = reinterpret_cast<const int4*>(a.items);
    d.n_items = a.n_items;
    d.k_cache = reinterpret_cast<const half_t*>(a.k_cache);
    d.v_cache = reinterpret_cast<const half_t*>(a.v_cache);
    d.kv_old = a.kv_old;
    d.cap = a.cap;
    d.scale_log2 = kLog2e / sqrtf(static_cast<float>(a.d));
    const int rep = a.nh / a.nkv;
    const bool decode_style = a.k_cache != nullptr && a.T <= 4 * a.B && (rep == 1 || rep == 2 || rep == 4 || rep == 8);
    if (decode_style) {
        // Few rows: cut the keys so that about four workgroups per CU stream the cache (needs the partial buffer
        // and pays one more launch, so only where the cache is long enough for the stream to matter).
        d.n_split = 1;
        d.part = a.partials;
        const int wgs = a.max_rows * a.nkv;
        if (a.partials && a.max_rows <= kAttnSplitRows && a.cap >= 1024 && wgs < 2 * attn_cus())
            d.n_split = std::min(kAttnSplitMax, (4 * attn_cus() + wgs - 1) / wgs);
        return a.d == 128 ? launch_decode_d<128>(d, rep, a.max_rows, a.nkv, stream)
                          : launch_decode_d<64>(d, rep, a.max_rows, a.nkv, stream);
    }
    const int items_max = (a.max_rows + kAttnBQ - 1) / kAttnBQ + a.B;
    d.items_max = items_max;
    const int levels = (a.max_rows + kAttnBQ - 1) / kAttnBQ;
    if (levels <= kItemLevels)
        hipLaunchKernelGGL(attn_items_kernel, dim3(1), dim3(256), 0, stream, a.cu_exec, a.B,
                           reinterpret_cast<int4*>(a.items), items_max, a.n_items, levels);
    else
        hipLaunchKernelGGL(attn_items_by_sequence_kernel, dim3(1), dim3(256), 0, stream, a.cu_exec, a.B,
                           reinterpret_cast<int4*>(a.items), items_max, a.n_items);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const dim3 grid(8 * ((items_max * a.nh + 7) / 8)), block(256);
    if (a.d == 128)
        hipLaunchKernelGGL(flash_prefill_kernel<128>, grid, block, 0, stream, d);
    else
        hipLaunchKernelGGL(flash_prefill_kernel<64>, grid, block, 0, stream, d);
    return hipGetLastError();
}

}  // namespace qtale
