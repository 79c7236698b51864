/*
 * qtale.h - C ABI of the MI355X (gfx950) library for QTALE's inference hot path:
 * the token-adaptive, weight-only int4 group-quantized decoder-layer forward.
 *
 * What the calls compute (paper: "QTALE: Quantization-Robust Token-Adaptive Layer Execution"):
 *   - every layer has a router g_l that scores each token of the layer's input x_l (Sec. 2.2, Eq. 2);
 *   - a token executes the layer iff its execute probability p_{l,0} = softmax(g_l(x_l))_0 is at least
 *     a threshold theta shared by all layers (Sec. 3.4, Eq. 9); theta = 0.5 is the arg-max rule of Eq. 2;
 *   - executed tokens take x_{l+1} = x_l + f_l(x_l) (Eq. 1), bypassed tokens keep x_{l+1} = x_l
 *     bit for bit (Eq. 3);
 *   - executed tokens are gathered into a dense matrix before the layer runs (App. B.2);
 *   - the layer's linears are weight-only group-quantized (4 bit, groups along the input dimension,
 *     Sec. 4.1); the execution ratio is changed at run time without touching the weights (Sec. 3.4).
 * The paper fixes neither the quantizer's arithmetic nor the inside of f_l; this library uses a
 * round-to-nearest asymmetric min/max quantizer with fp16 scale and integer zero-point, a linear
 * router whose output is the execute-minus-bypass logit z (p_{l,0} = sigmoid(z)), and a pre-norm
 * LLaMA block (RMSNorm, rotary embedding at the token's ORIGINAL absolute position with half-split
 * pairing, causal softmax attention among the EXECUTED tokens of the same sequence, SwiGLU MLP).
 *
 * Conventions
 *   - All data pointers are DEVICE pointers unless a comment says "host".  The caller owns every
 *     buffer; the library never allocates, frees or keeps device memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is enqueued
 *     on it and the calls return without waiting for the GPU.
 *   - Every call returns 0 (QTALE_OK) or a negative error code.  Arguments are validated before the
 *     first HIP call, so invalid arguments are reported even on a machine without a GPU.
 *   - Matrices are row-major.  "act dtype" is cfg->act_dtype (IEEE fp16 or bfloat16), the type of
 *     the residual stream and of the RMSNorm gains.  K/V caches are always fp16.
 */
#ifndef QTALE_H
#define QTALE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    QTALE_OK = 0,
    QTALE_ERR_INVALID_ARG = -1,        /* null pointer, NaN/out-of-range control value, negative size */
    QTALE_ERR_SHAPE = -2,              /* shapes inconsistent with each other or with the kernels' granularity */
    QTALE_ERR_UNSUPPORTED = -3,        /* bits/group/head_dim the kernels do not implement */
    QTALE_ERR_WORKSPACE_TOO_SMALL = -4,
    QTALE_ERR_HIP = -5                 /* a HIP runtime call or a kernel launch failed */
};

enum { QTALE_ACT_FP16 = 0, QTALE_ACT_BF16 = 1 };
enum { QTALE_MODE_RATIO = 0, QTALE_MODE_THRESHOLD = 1 };

const char* qtale_strerror(int code);

/* ---- control state: which tokens execute (Sec. 3.4) --------------------------------------------
 * A context only holds the selection mode and its value.  Default: ratio mode, r = 1. */
typedef struct qtale_ctx qtale_ctx;
int qtale_create(qtale_ctx** out);
int qtale_destroy(qtale_ctx* ctx);

/* Ratio mode: in every layer of every later forward call exactly k = floor(r*T + 1/2) of the call's T
 * tokens execute, namely the k with the highest router score (equal scores: lower token index first).
 * r in [0,1]; NaN or out of range -> QTALE_ERR_INVALID_ARG.  Touches no weight buffer. */
int qtale_set_exec_ratio(qtale_ctx* ctx, float r);
/* Threshold mode (Eq. 9 verbatim): a token executes iff sigmoid(z) >= theta, decided as
 * z >= fp32(ln(theta/(1-theta))).  theta <= 0 executes every token, theta >= 1 none; NaN -> error. */
int qtale_set_threshold(qtale_ctx* ctx, float theta);
int qtale_get_control(const qtale_ctx* ctx, int* mode /*host*/, float* value /*host*/);

/* ---- quantized weights (Sec. 4.1: weight-only, groups along the input dimension) ----------------
 * W is [N][K] (out x in), fp32.  Per (row n, group g of `group` consecutive k; the last group may be
 * short): lo = min(0,min W), hi = max(0,max W), scale = fp16((hi-lo)/(2^bits-1)) (1.0 if that is 0 or
 * not finite), zero = clamp(rint(-lo/scale)), code = clamp(rint(W/scale)+zero); IEEE fp32 arithmetic,
 * round-half-even.  Dequantized weight: (code - zero) * scale.
 *   codes     bits = 4: [N][ceil(K/8)] uint32, nibble j of word w = code of k = 8*w + j;
 *             bits = 3: [N][3*ceil(K/32)] uint32, the row's codes as one little-endian bit stream, code k
 *             at bits 3k..3k+2 (32 codes fill three words); row tails padded with code 0
 *   scales    [N][ceil(K/group)] fp16 bit patterns
 *   zeros     [N][ceil(K/group)] fp16 bit patterns of the integer zero-point
 *   prepacked the kernels' private copy (codes reordered for the matrix-core operand layout plus
 *             scale/zero pairs), qtale_prepacked_bytes() bytes, 16-byte aligned; may be NULL here.
 * Supported: bits in {4, 3} (Sec. 4.1 evaluates both) and 2 (for mixed 2-/4-bit stacks: 16 codes per word,
 * bit pair j of word w = code of k = 16*w + j); group in {32, 64, 128}; K % 8 == 0.  Else
 * QTALE_ERR_UNSUPPORTED / _SHAPE.
 * The GEMM entry points (forward calls, qtale_linear_w4a16, qtale_swiglu_w4a16) also need N % 8 == 0. */
size_t qtale_prepacked_bytes(int N, int K, int bits, int group);
int qtale_quantize(const float* W, int N, int K, int bits, int group,
                   uint32_t* codes, uint16_t* scales, uint16_t* zeros,
                   void* prepacked /*nullable*/, void* stream);
/* Builds `prepacked` from canonical codes/scales/zeros (e.g. weights quantized elsewhere). */
int qtale_prepack(const uint32_t* codes, const uint16_t* scales, const uint16_t* zeros,
                  int N, int K, int bits, int group, void* prepacked, void* stream);

typedef struct {
    const uint32_t* codes;      /* canonical; not read by the forward calls, may be NULL */
    const uint16_t* scales;     /* canonical; may be NULL */
    const uint16_t* zeros;      /* canonical; may be NULL */
    const void* prepacked;      /* required by the forward calls */
    int N, K;
} qtale_qlinear;

typedef struct {
    int hidden, n_heads, n_kv_heads, head_dim, inter;   /* head_dim must be 64 or 128 */
    int bits;                                           /* 4, 3 or 2: default code width of the seven linears */
    int group;                                          /* 32, 64 or 128 */
    int act_dtype;                                      /* QTALE_ACT_FP16 | QTALE_ACT_BF16 */
    float rms_eps;                                      /* e.g. 1e-5 */
    float rope_base;                                    /* e.g. 10000 */
} qtale_layer_cfg;

typedef struct {
    qtale_qlinear q, k, v, o, gate, up, down;  /* q [nh*d][H], k,v [nkv*d][H], o [H][nh*d], gate,up [I][H], down [H][I] */
    const void* norm1;                         /* [hidden], act dtype: gain of the pre-attention RMSNorm */
    const void* norm2;                         /* [hidden], act dtype: gain of the pre-MLP RMSNorm */
    const float* router_w;                     /* [hidden] fp32: z_t = router_w . x_t + router_b */
    float router_b;
    /* Optional two-output MLP router (Sec. 2.2), used instead of router_w/router_b when router_hidden > 0:
     * u = relu(W1 x_t + b1), (l_e, l_b) = W2 u + b2, z_t = l_e - l_b (p_0 of Eq. 9 = sigmoid(z_t)); fp64 sums,
     * one rounding to fp32.  The paper gives no depth, width or activation: one hidden ReLU layer is this
     * library's reading.  router_hidden in 1..256; router_w may then be NULL. */
    int router_hidden;                         /* R; 0 = linear router */
    const float* router_w1;                    /* [R][hidden] fp32 */
    const float* router_b1;                    /* [R] fp32 */
    const float* router_w2;                    /* [2][R] fp32: row 0 execute logit, row 1 bypass logit */
    const float* router_b2;                    /* [2] fp32 */
    int bits;                                  /* code width of THIS layer's linears; 0 = cfg->bits (mixed-precision stacks) */
} qtale_layer_weights;

/* Per-layer K/V cache holding entries of EXECUTED tokens only (a bypassed token produces no key or
 * value at that layer).  k_cache/v_cache: [B][n_kv_heads][cap][head_dim] fp16 (the entries of one sequence
 * and head are contiguous: decode attention streams them at the full memory rate); kv_len [B] int32 device:
 * entries already present per sequence.  A forward call appends the executed tokens of sequence b (keys
 * after rotary embedding) at kv_len[b].. and adds their number to kv_len[b].  The caller should guarantee
 * kv_len[b] + (tokens of sequence b in the call) <= cap.  If it does not, the entries that would not fit are
 * dropped (the newest tokens of the call), kv_len[b] stops at cap, and those tokens' own queries attend to the cap
 * entries present: kv_len[b] == cap after a call is the caller's sign that the cache is full. */
typedef struct {
    void* k_cache;
    void* v_cache;
    int32_t* kv_len;
    int cap;
} qtale_kv;

/* Bytes of scratch a forward call with at most max_tokens tokens in max_seqs sequences needs.
 * Returns 0 for an invalid cfg. */
size_t qtale_workspace_bytes(const qtale_layer_cfg* cfg, int max_tokens, int max_seqs);

/* One token-adaptive layer (Eq. 1, 3, 9; App. B.2), in place on x.
 *   x            [T][hidden] act dtype; rows of bypassed tokens are not written
 *   seq_offsets  [B+1] int32: tokens seq_offsets[b]..seq_offsets[b+1]-1 form sequence b, in order;
 *                seq_offsets[0] = 0, seq_offsets[B] = T
 *   positions    [T] int32: absolute position of every token (for the rotary embedding)
 *   kv           nullable: NULL = the call's tokens are the whole context (pure prefill)
 *   sel_idx      nullable [T] int32 out: ascending indices of the executed tokens (first *sel_count valid)
 *   sel_count    nullable [1] int32 out
 *   scores       nullable [T] fp32 out: router scores z
 *   workspace    >= qtale_workspace_bytes(cfg, T, B) bytes, 256-byte aligned
 * T = 0 is a no-op.  With k = 0 executed tokens no kernel touches x. */
int qtale_layer_forward(qtale_ctx* ctx, const qtale_layer_cfg* cfg, const qtale_layer_weights* w,
                        void* x, int T, const int32_t* seq_offsets, int B, const int32_t* positions,
                        const qtale_kv* kv, int32_t* sel_idx, int32_t* sel_count, float* scores,
                        void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): qtale_layer_forward with the workspace taken from an array inside the library instead
 * of a caller buffer.  Same arguments, same kernels and bit-identical results; the call allocates and frees
 * nothing.  The array is QTALE_STATIC_SCRATCH_BYTES large (enough for a decode step of 128 one-token sequences
 * at hidden 5120 / 40 heads / SwiGLU 13824, or about 250 prefill tokens at hidden 4096 / SwiGLU 11008) and every
 * GPU the library runs on holds one copy until the process ends.  A call whose workspace
 * (qtale_workspace_bytes(cfg, T, B)) is larger returns QTALE_ERR_WORKSPACE_TOO_SMALL before any GPU work.
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU (different streams or threads) race;
 * serialize them.  Returns QTALE_ERR_INVALID_ARG while per-kernel profiling is enabled. */
#define QTALE_STATIC_SCRATCH_BYTES (40u << 20)
size_t qtale_static_scratch_bytes(void);
int qtale_layer_forward_static(qtale_ctx* ctx, const qtale_layer_cfg* cfg, const qtale_layer_weights* w,
                               void* x, int T, const int32_t* seq_offsets, int B, const int32_t* positions,
                               const qtale_kv* kv, int32_t* sel_idx, int32_t* sel_count, float* scores,
                               void* stream);

/* n_layers layers in sequence with the context's single control value (one global knob, Sec. 3.4).
 *   layers       host array [n_layers]
 *   kv_per_layer host array [n_layers], nullable
 *   sel_idx      nullable [n_layers][T]; sel_count nullable [n_layers]; scores nullable [n_layers][T]
 *   dbg_hidden   nullable [n_layers][T][hidden] act dtype: receives the INPUT of every layer */
int qtale_stack_forward(qtale_ctx* ctx, const qtale_layer_cfg* cfg, const qtale_layer_weights* layers,
                        int n_layers, void* x, int T, const int32_t* seq_offsets, int B,
                        const int32_t* positions, const qtale_kv* kv_per_layer,
                        int32_t* sel_idx, int32_t* sel_count, float* scores, void* dbg_hidden,
                        void* workspace, size_t workspace_bytes, void* stream);

/* ---- single steps of the path, exposed for tests and per-kernel measurement --------------------- */

/* Router scores and selection alone (steps 1-3 of a layer): z, ascending idx, count. */
int qtale_router_select(qtale_ctx* ctx, int act_dtype, const void* x, int T, int hidden,
                        const float* router_w, float router_b,
                        const int32_t* seq_offsets, int B,
                        float* scores /*[T]*/, int32_t* sel_idx /*[T]*/, int32_t* sel_count /*[1]*/,
                        int32_t* cu_exec /*nullable [B+1]: executed tokens before each sequence*/,
                        void* stream);

/* ---- threshold calibration (Sec. 3.4: two-phase grid search for the global theta) --------------------
 * Candidates theta_n = fp32(n/100), n = 1..50 (the search range (0, 0.5]).  Coarse pass over n = 5, 10,
 * ..., 50, then the not yet evaluated n within 4 steps of the best coarse point; the result is the evaluated
 * n whose average execution ratio R_avg is closest to target_ratio (ties: the larger theta).  The paper's
 * objective is a task metric on calibration data; here it is the execution ratio itself.
 * Both calls synchronize `stream`, allocate nothing, and on success leave ctx in threshold mode at the theta
 * found (as qtale_set_threshold would); on failure the control value is unchanged.
 *   scratch    device, qtale_calibration_scratch_bytes(n_layers) bytes (n_layers = 0 for the score form)
 *   theta, ratio  host out (nullable): theta found and its R_avg
 *   table      host out (nullable) [50]: R_avg of every evaluated candidate at index n-1, NaN elsewhere */
#define QTALE_THETA_GRID 50
size_t qtale_calibration_scratch_bytes(int n_layers);
/* Scores taken as fixed: scores is a device array of n fp32 router scores (e.g. [L][T] written by a forward
 * call); R_avg(theta) = fraction of them with sigmoid(z) >= theta, decided as in qtale_set_threshold. */
int qtale_calibrate_threshold_from_scores(qtale_ctx* ctx, const float* scores, int64_t n, float target_ratio,
                                          void* scratch, float* theta, float* ratio, float* table, void* stream);
/* R_avg measured: for every candidate the stack runs in threshold mode on the calibration batch (skipping
 * changes the hidden states later routers see) and R_avg = executed (layer, token) pairs / (n_layers * T).
 * x_calib [T][hidden] act dtype is only read; x_work (same size) is overwritten.  No K/V cache is used.
 * Other arguments as in qtale_stack_forward. */
int qtale_calibrate_threshold(qtale_ctx* ctx, const qtale_layer_cfg* cfg, const qtale_layer_weights* layers,
                              int n_layers, const void* x_calib, void* x_work, int T,
                              const int32_t* seq_offsets, int B, const int32_t* positions, float target_ratio,
                              void* scratch, void* workspace, size_t workspace_bytes,
                              float* theta, float* ratio, float* table, void* stream);

/* Scores of the two-output MLP router alone (see qtale_layer_weights): scores[t] for T tokens. */
int qtale_router_mlp_scores(int act_dtype, const void* x, int T, int hidden, const float* w1, const float* b1,
                            const float* w2, const float* b2, int router_hidden, float* scores /*[T]*/, void* stream);

/* out[M][N] (fp16) = A[M][K] (fp16) x dequant(W)^T for one quantized linear (matrix-core GEMM on 4-bit or
 * 3-bit codes, `bits`/`group` as given to qtale_quantize for this matrix). */
int qtale_linear_w4a16(const qtale_qlinear* w, int bits, int group, const void* A, int M, void* out, void* stream);

/* act[M][I] (fp16) = silu(A Wgate^T) * (A Wup^T): the fused gate/up GEMM of the SwiGLU MLP. */
int qtale_swiglu_w4a16(const qtale_qlinear* gate, const qtale_qlinear* up, int bits, int group,
                       const void* A, int M, void* out, void* stream);

/* ---- HIP graph of one stack forward (launch-overhead removal, App. B.2 future work) -------------------
 * qtale_graph_capture_stack records the kernels of ONE qtale_stack_forward call with exactly these
 * arguments (no dbg_hidden) into a HIP graph and instantiates it; nothing executes during capture.
 * Every pointer and the control value of ctx at capture time are baked in (in ratio mode the launch shapes
 * depend on the ratio): to step a decode loop the caller rewrites x, positions and the caches' contents in
 * place between launches; per-sequence cache lengths advance on the device as in the eager call.  After
 * qtale_set_exec_ratio / qtale_set_threshold a new graph must be captured.  Fails with
 * QTALE_ERR_INVALID_ARG while per-kernel profiling is enabled.
 * qtale_graph_launch enqueues one replay on `stream`; replays of one graph must not overlap. */
typedef struct qtale_graph qtale_graph;
int qtale_graph_capture_stack(qtale_ctx* ctx, const qtale_layer_cfg* cfg, const qtale_layer_weights* layers,
                              int n_layers, void* x, int T, const int32_t* seq_offsets, int B,
                              const int32_t* positions, const qtale_kv* kv_per_layer /*nullable*/,
                              int32_t* sel_idx /*nullable*/, int32_t* sel_count /*nullable*/,
                              float* scores /*nullable*/, void* workspace, size_t workspace_bytes,
                              qtale_graph** graph /*host out*/);
int qtale_graph_launch(qtale_graph* graph, void* stream);
void qtale_graph_destroy(qtale_graph* graph);

/* Per-kernel timing with HIP events recorded on the forward call's stream.  While enabled, every
 * layer/stack forward brackets its kernels with events; qtale_profile_read waits for them and
 * returns, per kernel class, accumulated milliseconds and launch counts since the last read.
 * Classes: 0 router, 1 select, 2 norm1, 3 qkv gemm, 4 rope+append, 5 attention, 6 o gemm, 7 norm2,
 * 8 gate/up gemm, 9 down gemm.  Profiling adds event overhead; leave it off when timing whole steps. */
enum { QTALE_PROF_CLASSES = 10 };
int qtale_profile_enable(qtale_ctx* ctx, int on);
int qtale_profile_read(qtale_ctx* ctx, double* ms /*host [QTALE_PROF_CLASSES]*/,
                       int64_t* launches /*host [QTALE_PROF_CLASSES]*/);

#ifdef __cplusplus
}
#endif
#endif /* QTALE_H */
