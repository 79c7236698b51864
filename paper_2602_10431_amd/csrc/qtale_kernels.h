// Host-side launchers of the gfx950 kernels (internal; the public boundary is include/qtale.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace qtale {

struct PrepackDims {
    int NF, KT, NGP;
    size_t code_bytes, sz_bytes;
};
PrepackDims prepack_dims(int N, int K, int group, int bits);

hipError_t launch_quantize(const float* W, int N, int K, int bits, int group, uint32_t* codes,
                           uint16_t* scales, uint16_t* zeros, hipStream_t stream);
hipError_t launch_prepack(const uint32_t* codes, const uint16_t* scales, const uint16_t* zeros, int N,
                          int K, int bits, int group, void* prepacked, hipStream_t stream);

// ---- router + selection --------------------------------------------------------------------
hipError_t launch_router_score(const void* x, int bf16, int T, int H, const float* w, float b,
                               float* z, hipStream_t stream);

// Two-output MLP router: z_t = (W2 relu(W1 x_t + b1) + b2)[0] - (...)[1]; W1 [R][H], b1 [R], W2 [2][R], b2 [2] fp32.
hipError_t launch_router_mlp(const void* x, int bf16, int T, int H, const float* W1, const float* b1, const float* W2,
                             const float* b2, int R, float* z, hipStream_t stream);

struct SelectArgs {
    const float* z;            // [T]
    int T;
    int mode;                  // 0 ratio, 1 threshold
    int k;                     // ratio mode: number of tokens to execute
    float z_thr;               // threshold mode
    const int32_t* seq_offsets;  // [B+1]
    int B;
    int32_t* idx;              // [T] out
    int32_t* count;            // [1] out
    int32_t* cu_exec;          // [B+1] out (nullable)
    int32_t* row_seq;          // [T] out: sequence of each executed row (nullable)
    int32_t* kv_len;           // [B] in/out (nullable): advanced by the executed count of each sequence
    int32_t* kv_old;           // [B] out (nullable unless kv_len given): kv_len before the call
    int kv_cap;                // capacity of the cache behind kv_len (0 = unknown): kv_len is not advanced beyond it
    int32_t* idx_copy;         // nullable: second destination for idx (caller-visible output)
    int32_t* inv;              // nullable (small-call kernel only): [T] compact row of token t, -1 when bypassed
    int32_t* count_copy;       // nullable
};
hipError_t launch_select(const SelectArgs& a, hipStream_t stream);

// Decode-sized calls: selection / compaction and gather + RMSNorm 1 in one launch, reading the scores z [T] a router
// kernel has written; same outputs as launch_select + launch_gather_rmsnorm.  Only valid when
// fused_select_norm_fits(T, max_rows); max_rows > 0 is the host bound on executed rows.
bool fused_select_norm_fits(int T, int max_rows);
hipError_t launch_select_norm(const void* x, int bf16, int H, const float* z, const void* gain, float eps, void* out_f16,
                              const SelectArgs& s, int max_rows, hipStream_t stream);

// Decode-sized stacks: the last kernel of layer l (sum of the down-proj's K parts + residual + scatter, Eq. 1 and 3) also
// scores every token for layer l + 1 (Eq. 2, linear router; the same fp64 summation order as launch_router_score, on the
// values just stored).  inv [T] is the token -> compact row map of select_norm (-1 = bypassed: the row is only scored).
hipError_t launch_reduce_scatter_score(const float* part, int n_parts, int part_rows, const float* h, int H, const int32_t* inv,
                                       int T, void* x, int bf16, const float* w_next, float b_next, float* z_next,
                                       hipStream_t stream);

// Threshold calibration: bins[b] (kThetaGrid + 1 counters, cleared here) = number of scores that reach exactly
// b of the kThetaGrid ascending thresholds zthr_dev (device array).
constexpr int kThetaGrid = 50;
hipError_t launch_threshold_bins(const float* scores, long n, const float* zthr_dev, unsigned long long* bins,
                                 hipStream_t stream);

// ---- row operations ---------------------------------------------------------------------------
// n1[i] = fp16(rmsnorm(x[idx[i]]) * gain) for i < *count
hipError_t launch_gather_rmsnorm(const void* x, int bf16, int H, const int32_t* idx, const int32_t* count,
                                 int max_rows, const void* gain, float eps, void* out_f16, hipStream_t stream);
// n2[i] = fp16(rmsnorm(h[i]) * gain), h fp32
hipError_t launch_rmsnorm_f32(const float* h, int H, const int32_t* count, int max_rows, const void* gain,
                              int gain_bf16, float eps, void* out_f16, hipStream_t stream);

struct RopeArgs {
    void* qkv;                 // [rows][(nh+2nkv)*d] fp16, q and k rotated in place
    int nh, nkv, d;
    float base;
    const int32_t* idx;        // compact row -> token
    const int32_t* positions;  // [T]
    const int32_t* count;
    int max_rows;
    // optional cache append
    void* k_cache; void* v_cache; int cap;
    const int32_t* row_seq; const int32_t* cu_exec; const int32_t* kv_old;
};
hipError_t launch_rope_append(const RopeArgs& a, hipStream_t stream);

// Consumers of the decode GEMM's partial tiles (part = fp32 [n_parts][max_rows][H], added in part order):
//   h[i] = x[idx[i]] + sum(part[.][i]);  n2[i] = fp16(rmsnorm(h[i]) * gain)          (after the o-proj)
hipError_t launch_reduce_rmsnorm(const float* part, int n_parts, const void* x, int bf16, const int32_t* idx, int H,
                                 const int32_t* count, int max_rows, const void* gain, float eps, float* h,
                                 void* out_f16, hipStream_t stream);
//   x[idx[i]] = act(h[i] + sum(part[.][i]))                                           (after the down-proj)
hipError_t launch_reduce_scatter(const float* part, int n_parts, const float* h, int H, const int32_t* idx,
                                 const int32_t* count, int max_rows, void* x, int bf16, hipStream_t stream);

// ---- W4A16 / W3A16 GEMM ---------------------------------------------------------------------------------
enum GemmEpilogue { EPI_STORE_F16 = 0, EPI_RESID_F32 = 1, EPI_SWIGLU_F16 = 2, EPI_RESID_SCATTER = 3,
                    EPI_PARTIAL_F32 = 4 };   // fp32 partial tiles [parts][M_max][ldo], decode kernel only

struct GemmWeights {
    const void* prepacked;
    int N, K;
};

struct GemmArgs {
    const void* A;             // [M][K] fp16
    const int32_t* count;      // device row count (nullable: use M_max)
    int M_max;                 // host upper bound of rows
    int rows_exact;            // nonzero: the row count equals M_max (ratio mode); zero: M_max is a bound, the count is read on the device
    int K;
    int group;
    int bits;                  // 4 or 3
    int n_w;                   // number of weight matrices: 1, 2 (gate/up interleaved), 3 (q|k|v concatenated)
    GemmWeights w[3];
    int epilogue;
    void* out;                 // STORE/SWIGLU: fp16 [M][ldo]; RESID_F32: fp32 [M][ldo]; RESID_SCATTER: act dtype x [T][ldo]
    int ldo;
    const void* resid;         // RESID_F32: x (act dtype, rows via idx); RESID_SCATTER: h fp32 [M][ldo]
    const int32_t* idx;        // compact row -> token row (RESID_F32 reads, RESID_SCATTER writes)
    int bf16;                  // act dtype of x
    // Decode steps (M_max <= kGemmPartRows) with a RESID_* epilogue: when `part` is given the GEMM may cut K across
    // workgroups and write fp32 partial tiles [*n_parts][M_max][ldo] there INSTEAD of applying its epilogue; the
    // caller then runs the consumer that adds the parts (launch_reduce_rmsnorm / launch_reduce_scatter).
    float* part;               // nullable: room for kGemmPartMax x M_max x ldo floats
    int* n_parts;              // host out, required with `part`: 0 = epilogue applied as usual, else parts written
};
constexpr int kGemmPartRows = 64;
constexpr int kGemmPartMax = 4;
hipError_t launch_gemm_w4a16(const GemmArgs& a, hipStream_t stream);

// ---- attention over executed tokens ---------------------------------------------------------------
struct AttnArgs {
    const void* qkv;           // [rows][(nh+2nkv)*d] fp16 (q rotated, k rotated, v)
    void* out;                 // [rows][nh*d] fp16
    int nh, nkv, d;
    const int32_t* count;
    int max_rows;              // host bound on executed rows
    int B;
    const int32_t* cu_exec;    // [B+1]
    const int32_t* row_seq;    // [rows]
    // cache (nullable): when given, keys/values are read from the cache only (new rows were appended)
    const void* k_cache; const void* v_cache; int cap;
    const int32_t* kv_old;     // [B]
    int T;                     // tokens in the call
    void* items;               // scratch: (max_rows / kAttnBQ + B + 1) x int4 work list of the prefill kernel, 16-byte aligned
    int32_t* n_items;          // scratch [1]
    float* partials;           // scratch (nullable): min(max_rows, kAttnSplitRows) x nh x kAttnSplitMax x (d + 2) fp32,
                               // lets the decode kernel cut long caches into key ranges when there are few rows
};
constexpr int kAttnBQ = 128;   // executed rows per prefill-attention workgroup
constexpr int kAttnSplitRows = 128;   // decode attention splits the keys only up to this many rows
constexpr int kAttnSplitMax = 8;      // and into at most this many ranges
hipError_t launch_attention(const AttnArgs& a, hipStream_t stream);

}  // namespace qtale
