/*
 * libsla2 - SLA2 attention (forward pass, and its backward pass) on MI355X (gfx950), C ABI.
 *
 * The operator is  O = SLA2(Q, K, V, k%, R, alpha)  of the paper
 * "SLA2: Sparse-Linear Attention with Learnable Routing and QAT":
 *
 *   O   = alpha (.) O_s + (1 - alpha) (.) O_l                      (Eq. 13)
 *   O_s = softmax(Q K^T / sqrt(d) restricted to M = 1) V           (Eq. 14)
 *   O_l = norm(phi(Q) phi(K)^T (.) (1 - M)) V,  phi = softmax_d    (Eq. 14)
 *   M   = expansion of M_c = Top-k(k%, proj_q(pool Q) proj_k(pool K)^T)   (Eq. 15-16)
 *
 * computed block-wise as in the paper's forward algorithm (Alg. 2), with K
 * first replaced by K - colmean(K).  sla2_backward returns the gradients of
 * Q, K, V and alpha (Alg. 3).
 *
 * Conventions for every entry point
 *   - q, k, v, out are DEVICE pointers to [B, H, N, d] tensors of params->dtype,
 *     contiguous unless params->in_stride / out_stride say otherwise; router_w, alpha, block_idx, lse, workspace are DEVICE
 *     pointers; params is a HOST pointer.  All memory is owned by the caller;
 *     the library allocates nothing, frees nothing and never synchronises.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*;
 *     NULL = the default stream) and completes in stream order.
 *   - Arguments are validated on the host before anything is launched.  The
 *     return value is SLA2_OK (0) or a negative sla2_status; on an error no
 *     kernel has been launched (except SLA2_EHIP, which reports a failed
 *     launch).  No exceptions, no errno, no logging.
 *   - `workspace` must hold at least sla2_workspace_bytes(params) bytes and be
 *     256-byte aligned; its contents after a call are described by
 *     sla2_workspace_layout() and may be read by the caller (tests do).
 *     Calls that share a workspace must not overlap in time.
 */
#ifndef SLA2_H
#define SLA2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SLA2_OK = 0,
  SLA2_EINVAL = -1,       /* null pointer, non-positive size, topk_frac outside [0,1], bad enum */
  SLA2_EUNSUPPORTED = -2, /* a shape / mode combination the kernels do not cover (see sla2_params) */
  SLA2_EWORKSPACE = -3,   /* workspace null, misaligned or smaller than sla2_workspace_bytes() */
  SLA2_EALIAS = -4,       /* an output overlaps an input (or another output) */
  SLA2_EHIP = -5          /* a kernel launch failed */
} sla2_status;

typedef enum { SLA2_F32 = 0, SLA2_BF16 = 1 } sla2_dtype;   /* element type of q, k, v, out */

/* Precision of the sparse branch (Sec. 5 of the paper, "Quantization-aware training").
 *   SLA2_QUANT_NONE  Q K^T and P V in the storage type with fp32 accumulation.
 *   SLA2_QUANT_FP8   Q and the smoothed K as FP8 e4m3 (OCP; max 448) with one
 *                    scale per b_q x d block of Q and per b_kv x d block of K:
 *                    amax = max|x| over the block, stored value = rne(x * (448/amax)),
 *                    dequantisation scale amax/448, both divisions in fp32;
 *                    P rounded to e4m3 after scaling by 2^8; V kept in bf16;
 *                    the softmax denominator uses the un-rounded P.
 *                    Requires dtype = SLA2_BF16.
 *   SLA2_QUANT_INT8  as SLA2_QUANT_FP8 with Q and the smoothed K as symmetric INT8 codes
 *                    (the other low-bit format Sec. 5 names for Q K^T): stored value =
 *                    rne(x * (127/amax)) in [-127, 127], dequantisation scale amax/127;
 *                    the products of codes are exact integers.  P, V and the
 *                    denominator as in FP8 mode.  Requires dtype = SLA2_BF16.
 *   SLA2_QUANT_FP8_V as SLA2_QUANT_FP8, and the second product as Alg. 2 prints it,
 *                    dequant(quant(P) quant(V_j)): V_j in e4m3 with one scale per b_kv x d block
 *                    (same rule as for K, over the block's existing tokens), P V on the FP8
 *                    matrix product.  The linear branch keeps the input V.  Requires dtype = SLA2_BF16. */
typedef enum { SLA2_QUANT_NONE = 0, SLA2_QUANT_FP8 = 1, SLA2_QUANT_INT8 = 2, SLA2_QUANT_FP8_V = 3 } sla2_quant;

#define SLA2_FLAG_NO_SMOOTH_K 1u   /* skip K <- K - colmean(K) (first step of Alg. 2) */
#define SLA2_FLAG_SAVE_FOR_BACKWARD 2u   /* sla2_forward also keeps what sla2_backward needs (O^s, L, ...) in the
                                            workspace, and the workspace is sized for sla2_backward */

typedef struct sla2_params {
  int B, H, N, d;          /* batch, heads, tokens, head dim.  d in {64, 128}; N >= 1;
                              ceil(N / block_kv) <= 2048 */
  int block_q, block_kv;   /* b_q, b_kv of the paper: (64, 64) or (128, 64) */
  float topk_frac;         /* k% as a fraction in [0, 1]; each query block keeps
                              k = floor(topk_frac * T_n + 0.5) key/value blocks, T_n = ceil(N / block_kv) */
  int dtype;               /* sla2_dtype */
  int quant_mode;          /* sla2_quant */
  int router_w_per_head;   /* 0: router_w is [2, d, d], shared by all heads; 1: [H, 2, d, d] */
  int alpha_per_block;     /* 0: alpha is [H]; 1: alpha is [H, T_m], T_m = ceil(N / block_q)
                              (Alg. 2 takes one alpha per query block) */
  unsigned flags;          /* SLA2_FLAG_* */
  /* Element strides (batch, head, token) of q, k, v - which share one layout, e.g. the three
   * slices of a packed [B, N, 3, H, d] projection - and of out.  The head dimension is always
   * contiguous.  All three zero (the default) means the contiguous [B, H, N, d] layout,
   * i.e. (H*N*d, N*d, d).  A [B, N, H, d] tensor is (N*H*d, d, H*d).  Every stride must be
   * positive, a multiple of 16 bytes, the token stride at least d and below 2^24 elements;
   * the caller guarantees that the strides describe memory it owns.  lse, block_idx and the
   * workspace arrays are not affected. */
  long long in_stride[3];
  long long out_stride[3];
} sla2_params;

/* Byte offsets, inside the workspace, of what a call leaves behind.  All are
 * multiples of 256.  "BH" = B*H, T_m / T_n = number of query / key blocks. */
typedef struct sla2_ws_layout {
  size_t q_sum;     /* double [BH, T_m, d]   sum of the rows of each query block            (Eq. 15 x block size) */
  size_t k_sum;     /* double [BH, T_n, d]   same for the raw K blocks */
  size_t k_mean;    /* double [BH, d]        colmean(K) (zeros with SLA2_FLAG_NO_SMOOTH_K)   (Alg. 2, smoothing) */
  size_t router_m;  /* double [1 or H, d, d] Wq Wk^T / sqrt(d): the two router projections folded into one matrix (Eq. 16) */
  size_t block_idx; /* int32  [BH, T_m, k]   ascending selected key/value blocks (M_c)      (Eq. 16) */
  size_t h_total;   /* float  [BH, d, d]     sum over all key blocks of (K^phi_j)^T V_j     (Alg. 2: h) */
  size_t z_total;   /* float  [BH, d]        sum over all key blocks of colsum(K^phi_j)     (Alg. 2: z) */
  size_t k_stats;   /* float  [BH, N]        per key token: lnZ = log sum_c exp(k'_c), k' = k - colmean(K); K^phi = exp(k' - lnZ) */
  size_t k_phi;     /* bf16   [BH, T_n, d/32, 4, 64, 8]  K^phi = softmax_d(K - colmean K) of each key block as matrix-core
                                                        operand fragments (bf16 path only): lane l of fragment (mt, ks)
                                                        holds channel 32 mt + l%32, tokens 16 ks + 8 (i/4) + 4 (l/32) + i%4, i = 0..7 */
  size_t z_blocks;  /* float  [BH, T_n, d]   z_j = colsum(K^phi_j) per key block (bf16 path only)        (Alg. 2: z) */
  size_t k_fp8;     /* uint8  [BH, T_n*block_kv, d]  e4m3 (FP8 mode) or two's-complement int8 (INT8 mode) codes of the
                       smoothed K; low-bit modes only; rows >= N are 0 */
  size_t k_scale;   /* float  [BH, T_n]      dequantisation scale of each key block (low-bit modes only) */
  size_t v_fp8;     /* uint8  [BH, T_n, d, block_kv]  e4m3 codes of V, one d x 64 tile per key block, transposed
                       (channel-major) with the 64 tokens of a row in the order the FP8 product consumes them:
                       byte 32 g + b of a row holds token 32 (b / 16) + 8 ((b % 16) / 4) + 4 g + b % 4
                       (g = 0, 1; b = 0..31).  SLA2_QUANT_FP8_V only; tokens >= N are 0 */
  size_t v_scale;   /* float  [BH, T_n]      dequantisation scale of each V block (SLA2_QUANT_FP8_V only) */
  size_t partial;   /* scratch for per-chunk partial sums of h and z */
  /* with SLA2_FLAG_SAVE_FOR_BACKWARD only (0 bytes otherwise): */
  size_t o_s;       /* dtype  [BH, N, d]     sparse-branch output O^s, before the mix of Eq. 13   (input of Alg. 3) */
  size_t o_l;       /* dtype  [BH, N, d]     linear-branch output O^l (fp32 tensors only; 0 bytes for bf16 tensors, whose
                       backward pass rebuilds what it needs of O^l from the state kept in `bwd`) */
  size_t lse;       /* float  [BH, N]        L_i of Alg. 2 (log-sum-exp of the kept scores; -inf when k = 0) */
  size_t bwd;       /* scratch of sla2_backward; for bf16 tensors sla2_forward also leaves the state of the
                       linear branch of every query block here (H_i^T as bf16, Z_i) */
  size_t total;     /* = sla2_workspace_bytes() */
} sla2_ws_layout;

/* Pure host functions.  Return 0 / fill `out` with zeros when params is invalid. */
size_t sla2_workspace_bytes(const sla2_params* params);
int sla2_workspace_layout(const sla2_params* params, sla2_ws_layout* out);
/* k of Eq. 16 for these parameters (floor(topk_frac * T_n + 0.5), clamped); negative sla2_status on error. */
int sla2_num_selected(const sla2_params* params);

/* Learnable router (Sec. 4, Eq. 15-16; router step of Alg. 2): mean-pool Q over
 * block_q tokens and K - colmean(K) over block_kv tokens (a ragged last block is
 * averaged over the tokens it has), project with router_w = [Wq | Wk] (each
 * [d_in, d_out] row-major fp32, proj(x) = x W, no bias), score
 * R = proj_q(Qbar) proj_k(Kbar)^T / sqrt(d) and keep, per query block, the k
 * largest scores; equal scores go to the lower block index.  The row softmax of
 * Alg. 2 is omitted, and so is the subtraction of colmean(K) inside the router
 * (it moves all scores of a row by the same amount): neither changes a row-wise
 * top-k.  All arithmetic is fp64 so that the selection matches an fp64
 * reference up to summation order.
 * block_idx: int32 [B, H, T_m, k], each row ascending.  With k = 0 nothing is written. */
int sla2_router(const sla2_params* params, const void* q, const void* k, const float* router_w,
                int32_t* block_idx, void* workspace, size_t workspace_bytes, void* hip_stream);

/* sla2_router for callers that cannot allocate device memory and hold no workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same result as sla2_router;
 * the intermediate arrays (fp64 block sums of Q and K, colmean(K), the folded router matrix - the part of
 * the workspace that precedes sla2_ws_layout.block_idx) live in an array of SLA2_STATIC_SCRATCH_BYTES that
 * is part of the library's device image: every GPU the library runs on holds it until the process ends.
 * The call allocates and frees nothing and never synchronises.  Parameters whose router arrays need more
 * than SLA2_STATIC_SCRATCH_BYTES (sla2_workspace_layout(params).block_idx bytes; 9.5 MB for B = 1, H = 12,
 * N = 32760, d = 128) are refused with SLA2_EWORKSPACE before anything is launched.  All calls on one GPU
 * share that GPU's array, which keeps the last call's contents (nothing in it has to start at zero):
 * calls that overlap in time on one GPU race - keep them on one stream or order them with events.
 * q, k, router_w, block_idx, hip_stream and the other errors as for sla2_router. */
#define SLA2_STATIC_SCRATCH_BYTES (32u << 20)
int sla2_router_static(const sla2_params* params, const void* q, const void* k, const float* router_w,
                       int32_t* block_idx, void* hip_stream);

/* SoftTop-k form of the router (Sec. 6: the differentiable operator that replaces Top-k in the
 * first training stage):  mask[b,h,i,j] = sigmoid(P_c[i,j] / tau + lambda_i), P_c the row softmax
 * of the router scores of Eq. 16 (with the 1/sqrt(d) of Alg. 2), lambda_i found by bisection so that
 * row i sums to k = sla2_num_selected(params); k = 0 gives zeros, k = T_n ones.  fp64 inside.
 *   q, k, router_w  as for sla2_router;  tau > 0 (the paper uses 0.1)
 *   mask_out        DEVICE float [B, H, T_m, T_n], written
 * Same workspace, stream and error conventions as sla2_router; SLA2_EINVAL if tau is not positive. */
int sla2_router_soft(const sla2_params* params, const void* q, const void* k, const float* router_w,
                     float tau, float* mask_out, void* workspace, size_t workspace_bytes, void* hip_stream);

/* The whole forward pass (Alg. 2; Eq. 13-16): router as above, then for every
 * query block the sparse branch over its selected key/value blocks in ascending
 * order (online softmax), the linear branch over the others - formed as the
 * per-head total of h_j, z_j minus the selected blocks - and the alpha mix.
 * alpha values are used as given (the caller keeps them in [0,1]).  A query
 * block with no selected block has O_s = 0; one with every block selected has
 * O_l = 0.  The subtraction is taken in fp32 on fp32 totals; when all but a few
 * blocks are selected (k close to T_n) the linear branch is the small difference
 * of two large sums and carries their rounding (bf16 tensors: the selected blocks'
 * h_j are rebuilt from bf16 operands) - measured at k = T_n - 1 with a one-token
 * last block it stays inside the tolerances stated for each precision mode.
 * out:               [B, H, N, d] of params->dtype.
 * block_idx_or_null: if non-null receives the mask as in sla2_router.
 * lse_or_null:       if non-null receives float [B, H, N]: L = m + log l of the
 *                    sparse branch (the L_i of Alg. 2), -inf when k = 0. */
int sla2_forward(const sla2_params* params, const void* q, const void* k, const void* v,
                 const float* router_w, const float* alpha, void* out,
                 int32_t* block_idx_or_null, float* lse_or_null,
                 void* workspace, size_t workspace_bytes, void* hip_stream);

/* Backward pass (Alg. 3 of the appendix, plus the steps it leaves to automatic differentiation: phi,
 * the smoothing of K, the mix of Eq. 13): gradients of q, k, v and alpha for the block mask of the
 * matching forward call (hard Top-k passes no gradient to the router, Sec. 6).  Taken from the
 * original q, k, v whatever quant_mode the forward ran in (Sec. 5): fp32 arithmetic for fp32 tensors;
 * for bf16 tensors the products run on the matrix cores (bf16 operands, fp32 accumulation) and
 * everything between them is fp32.
 *   params     the params of the forward call, SLA2_FLAG_SAVE_FOR_BACKWARD set
 *   workspace  the workspace of that forward call, untouched since: it holds the block lists, the
 *              per-token and per-head statistics of K, O^s, O^l and L
 *   q, k, v, alpha   as in the forward call;  dout: gradient of out, layout of out (out_stride)
 *   dq, dk, dv       written; element type and layout of q, k, v (in_stride); must not overlap
 *                    each other or any input (they may be the slices of one packed [B, N, x, H, d]
 *                    buffer: interleaved, sharing no element)
 *   dalpha           DEVICE float [H] or [H, T_m] (alpha_per_block), written
 * Deterministic: fixed summation orders; the only atomic is an order-independent OR on LDS words.  Errors as sla2_forward; SLA2_EINVAL without the flag. */
int sla2_backward(const sla2_params* params, const void* q, const void* k, const void* v, const float* alpha,
                  const void* dout, void* dq, void* dk, void* dv, float* dalpha,
                  void* workspace, size_t workspace_bytes, void* hip_stream);

/* Dense attention softmax(Q K^T / sqrt(d)) V with the same tile machinery: the
 * comparator the paper measures speed-ups against (Sec. 9.1: C = 4 N^2 d).
 * Uses B, H, N, d, dtype of params (dtype must be SLA2_BF16); needs no workspace. */
int sla2_dense_forward(const sla2_params* params, const void* q, const void* k, const void* v,
                       void* out, void* hip_stream);

/* Per-kernel timing for benchmarks (not part of the operator).  While no profile is open the other entry
 * points share no mutable host state and may be called from several threads; between sla2_profile_begin
 * and sla2_profile_end all calls must come from one thread.
 * The forward pass is a fixed sequence of kernels ("stages").  Between sla2_profile_begin and
 * sla2_profile_end every launch of a stage whose bit is set in stage_mask is bracketed by two
 * hipEventRecord calls on the caller's stream, for at most max_calls calls of sla2_forward /
 * sla2_router / sla2_dense_forward / sla2_backward; the events are created in sla2_profile_begin, so the
 * calls in between still allocate nothing.  sla2_profile_end synchronises on the recorded
 * events, adds up the elapsed milliseconds and the number of launches per stage into the two
 * HOST arrays (each SLA2_STAGE_COUNT long) and destroys the events.
 * Returns SLA2_OK, SLA2_EINVAL (bad arguments / begin without end) or SLA2_EHIP. */
typedef enum {
  SLA2_STAGE_BLOCK_SUMS = 0,  /* pooling sums of Q and K blocks; router weights folded   (Eq. 15-16) */
  SLA2_STAGE_TOPK = 1,        /* projection, scores, row-wise top-k; colmean(K)   (Eq. 16; Alg. 2, smoothing) */
  SLA2_STAGE_KV_STATE = 2,    /* K^phi, partial h and z, low-bit codes of K (Alg. 2: K^phi, h, z) */
  SLA2_STAGE_KV_TOTAL = 3,    /* per-head totals of h and z */
  SLA2_STAGE_ATTN = 4,        /* sparse + linear branch + mix              (Alg. 2 block loop, Eq. 13) */
  SLA2_STAGE_DENSE = 5,       /* dense attention comparator */
  SLA2_STAGE_BWD_LISTS = 6,   /* sla2_backward: the block mask as bits, per key block the list of its query blocks */
  SLA2_STAGE_BWD_Q = 7,       /* query-side kernel: D^s, D^l, dQ, dH_i, dZ_i, d alpha parts          (Alg. 3) */
  SLA2_STAGE_BWD_KV = 8,      /* key-side kernel: dK', dV                                             (Alg. 3) */
  SLA2_STAGE_BWD_REST = 9,    /* totals of dH_i, dZ_i; dK = dK' - colmean(dK'); d alpha               */
  SLA2_STAGE_COUNT = 10
} sla2_stage;
int sla2_profile_begin(unsigned stage_mask, int max_calls);
/* The same, bracketing only calls 1, 1 + every, 1 + 2 every, ... (at most max_calls of them), for
 * callers that want a few samples out of a long loop.  every >= 1. */
int sla2_profile_begin_sampled(unsigned stage_mask, int max_calls, int every);
int sla2_profile_end(double* stage_ms, int* stage_launches);

const char* sla2_strerror(int status);
int sla2_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SLA2_H */
