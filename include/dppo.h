/*
 * dppo.h -- C ABI of the DPPO per-token divergence trust-region loss for AMD MI355X (gfx950).
 *
 * One call evaluates, for T response tokens (rows) over a vocabulary of V entries, the policy
 * loss of Divergence Proximal Policy Optimization ("Rethinking the Trust Region in LLM
 * Reinforcement Learning", Sec. 4.3-4.4, App. C.1):
 *
 *   log pi(.|s_t)  = log-softmax of the trainer logits z[t, 0..V)                 (Sec. 3)
 *   r_t            = pi(a_t|s_t) / mu(a_t|s_t),  mu = the ROLLOUT policy          (Eq. ppo-clip,
 *                                                                                  Sec. 5.2)
 *   D_t            = Binary-TV | Binary-KL | Top-K-TV | Top-K-KL of (mu || pi)    (Eq. binary_tv,
 *                    over {a_t, rest} or over TopK(mu,K) U {a_t} U {other}         binary_kl,
 *                                                                                  topk_tv, topk_kl)
 *                    or, given the rollout policy's full logits, the exact full-vocabulary
 *                    TV / KL those approximate                                     (App. B)
 *   M_t            = 0 iff D_t > delta and ((A_t>0 and r_t>1) or (A_t<0 and r_t<1)), else 1
 *                                                                                  (Eq. dppo_obj)
 *   loss           = loss_scale * sum_t ( - M_t r_t A_t )      (the negated objective of
 *                                                               Eq. dppo_obj: to be minimised)
 *   grad_logits    = loss_scale * M_t A_t r_t (pi(j|s_t) - 1[j = a_t])   for every j < V
 *                    (Eq. unified_grad with C = infinity; M_t is a constant factor)
 *
 * The same call also evaluates the paper's baselines, which differ only in M_t and in the cap
 * C on the ratio (App. C.1): `mask_rule` selects the DPPO mask, the PPO/GRPO ratio-clip mask
 * or none, and `ratio_cap` replaces r_t by min(r_t, C) in the loss term and the gradient.
 *
 * All pointers are DEVICE pointers owned by the caller.  Inputs are read-only and, like the
 * outputs and the workspace, must stay valid until the work enqueued on `stream` has finished.
 * The library allocates nothing, never synchronises and never touches another stream; every
 * kernel is enqueued on `stream` (a hipStream_t passed as void*; NULL = the legacy default
 * stream; it must belong to the current device) and the call returns at once.  The return value reports host-side argument checks
 * and launch errors only.  Results are bitwise reproducible for identical arguments on the
 * same device.
 */
#ifndef DPPO_H
#define DPPO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DPPO_VERSION 301          /* major*10000 + minor*100 + patch                          */
#define DPPO_KMAX 1024            /* largest accepted K                                        */
#define DPPO_WORKSPACE_BYTES 65536  /* smallest workspace any call accepts                      */

/* Columns of the optional per-token diagnostics output [T, DPPO_NDIAG] (fp32): the health
 * metrics the paper monitors during training (App. F.1: mean |pi - mu| of the sampled token,
 * policy entropy) and the mass the top-K set covers (App. B.1), plus the ratio itself. */
#define DPPO_NDIAG 8
#define DPPO_DIAG_RATIO     0     /* r_t = pi(a_t) / mu(a_t)                                    */
#define DPPO_DIAG_LOGP      1     /* log pi(a_t|s_t)                                            */
#define DPPO_DIAG_ABS_DIFF  2     /* |pi(a_t) - mu(a_t)|                                        */
#define DPPO_DIAG_ENTROPY   3     /* -sum_j pi_j ln pi_j, nats                                  */
#define DPPO_DIAG_MASS_MU   4     /* mass mu puts on A' = TopK(mu,K) U {a_t} ({a_t} if Binary)  */
#define DPPO_DIAG_MASS_PI   5     /* mass pi puts on A'                                         */
                                  /* columns 6, 7: reserved, written as 0                      */

/* Which approximation of D(mu || pi) gates the update (Sec. 4.4).  KL is in nats. */
typedef enum {
  DPPO_BINARY_TV = 0,             /* |mu(a_t) - pi(a_t)|                       (Eq. binary_tv) */
  DPPO_BINARY_KL = 1,             /* Bernoulli KL on {a_t, not a_t}            (Eq. binary_kl) */
  DPPO_TOPK_TV   = 2,             /* 1/2 sum over A'' of |p_mu - p_pi|         (Eq. topk_tv)   */
  DPPO_TOPK_KL   = 3,             /* sum over A'' of p_mu ln(p_mu / p_pi)      (Eq. topk_kl)   */
  /* The exact divergences the four above lower-bound (App. B), over the whole vocabulary;
   * they need `mu_logits`.  KL has no floor: it is +inf where pi excludes (logit -inf) a token
   * that mu can sample. */
  DPPO_FULL_TV   = 4,             /* 1/2 sum_j |mu_j - pi_j|                   (App. B.1)      */
  DPPO_FULL_KL   = 5              /* sum_j mu_j ln(mu_j / pi_j)                (App. B.2)      */
} dppo_variant_t;

/* Which mask M_t gates the update (unified gradient form, App. C.1, Eq. unified_grad). */
typedef enum {
  DPPO_MASK_DIVERGENCE = 0,       /* DPPO: Eq. dppo_obj, on D_t of `variant` and `delta`          */
  DPPO_MASK_RATIO_CLIP = 1,       /* PPO / GRPO(-ClipHigher): 0 iff (A>0 and r > 1+eps_high) or  */
                                  /* (A<0 and r < 1-eps_low)                (App. C.1, App. E)  */
  DPPO_MASK_NONE       = 2        /* M_t = 1: PG-IS, PG-TIS / CISPO                (App. C.1)  */
} dppo_mask_rule_t;

typedef enum {
  DPPO_OK = 0,
  DPPO_ERR_NULL = 1,              /* a required pointer is NULL (mu_logits for DPPO_FULL_*)    */
  DPPO_ERR_SHAPE = 2,             /* T < 0, V < 1, ld < V, mu_ld < V (DPPO_FULL_*), or sizes   */
                                  /* beyond int32 row indexing                                 */
  DPPO_ERR_ALIGN = 3,             /* logits / mu_logits / grad_logits not 2-byte aligned,      */
                                  /* workspace not 8,                                          */
                                  /* diagnostics not 16                                        */
  DPPO_ERR_VARIANT = 4,           /* variant is not a dppo_variant_t                           */
  DPPO_ERR_K = 5,                 /* K < 0, K > DPPO_KMAX, or K > 0 without top-K pointers     */
                                  /* (with T > 0)                                              */
  DPPO_ERR_WORKSPACE = 6,         /* workspace NULL or smaller than dppo_workspace_bytes()     */
  DPPO_ERR_LAUNCH = 7,            /* the HIP runtime refused a launch (see hipGetLastError)    */
  DPPO_ERR_VALUE = 8              /* delta, loss_scale, eps_* or ratio_cap is NaN, eps_low not */
                                  /* in [0, 1), eps_high < 0, relax_alpha outside [0, 1],      */
                                  /* relax_sides or mask_rule unknown                          */
} dppo_status_t;

/* relax_sides */
#define DPPO_RELAX_HIGH 1u           /* eps_high = infinity for low-probability tokens          */
#define DPPO_RELAX_LOW 2u            /* eps_low = infinity (no lower bound) for them             */

/* flags */
#define DPPO_FLAG_FORCE_STREAMING 1u /* use the general kernels even where a register-resident
                                        one applies (testing / comparison)                     */
#define DPPO_FLAG_STATIC_ROWS 2u     /* never hand rows out at run time: every workgroup takes the
                                        rows its index fixes, one row at a time (testing /
                                        comparison)                                            */

typedef struct {
  /* ---- inputs ---- */
  const void*    logits;       /* bf16 [T, ld] row-major; only columns 0..V-1 are used.  (Where */
                               /* rows do not start on a 128-byte line a kernel may fetch the  */
                               /* whole aligned lines that hold a row: what such a line holds  */
                               /* beside the row - pad columns, a neighbouring row, up to 126  */
                               /* bytes in front of the first row, 2 behind the last - is      */
                               /* fetched and ignored, and never written in grad_logits.)      */
  int64_t        T;            /* rows (response tokens; the caller packs responses only)      */
  int64_t        V;            /* vocabulary size, 1 <= V < 2^31                               */
  int64_t        ld;           /* row pitch in elements, ld >= V (any value; fastest with      */
                               /* V % 8 == 0 and rows that start on 128-byte lines, i.e.       */
                               /* ld % 64 == 0 and a 128-byte aligned base; other rows of      */
                               /* 1024 .. 155585 entries still take a register-resident kernel */
                               /* if logits and grad_logits have the same address modulo 16,   */
                               /* a few per cent slower)                                       */
  const int32_t* sampled_ids;  /* [T] a_t.  An id outside [0, V) marks an ignored row:         */
                               /* divergence 0, mask 0, no loss term, zero gradient row        */
  const float*   mu_logp;      /* [T] log mu(a_t|s_t) as returned by the rollout engine        */
  const int32_t* mu_topk_ids;  /* [T, K] ids of mu's K most probable tokens (distinct per row; */
                               /* an id outside [0, V) is padding and is skipped; an id equal  */
                               /* to a_t is skipped, a_t always uses mu_logp).  NULL iff K = 0 */
  const float*   mu_topk_logp; /* [T, K] their log-probs under mu.  NULL iff K = 0             */
  int32_t        K;            /* 0 <= K <= DPPO_KMAX.  Used by the Top-K variants only; a     */
                               /* Top-K variant with K = 0 equals the Binary one               */
  int32_t        variant;      /* dppo_variant_t                                               */
  const float*   advantages;   /* [T] A_t per token (caller broadcasts sequence-level values)  */
  float          delta;        /* divergence threshold delta of Eq. dppo_obj                   */
  float          loss_scale;   /* multiplies loss and gradient, e.g. 1/T_total (the paper      */
                               /* leaves the minibatch normalisation to the trainer)           */
  int32_t        mask_rule;    /* dppo_mask_rule_t; 0 = the DPPO divergence mask.  D_t of      */
                               /* `variant` is computed and stored under every rule            */
  float          eps_low;      /* DPPO_MASK_RATIO_CLIP only: clip range [1-eps_low, 1+eps_high];*/
  float          eps_high;     /* "r > 1+eps" is evaluated as log pi - log mu > log(1+eps)     */
  float          ratio_cap;    /* C of Eq. unified_grad: the gradient weight is M min(r, C) A  */
                               /* (held constant) and the loss term -M min(r, C) A.            */
                               /* <= 0 or +inf: no cap (C = infinity, as DPPO uses)            */
  float          relax_alpha;  /* DPPO_MASK_RATIO_CLIP only (Sec. 6): for tokens whose ROLLOUT  */
                               /* probability mu(a_t) is below alpha the clip thresholds named */
                               /* by relax_sides are infinite.  0: none (GRPO); in [0, 1].     */
                               /* "mu(a_t) < alpha" is evaluated as log mu(a_t) < log alpha     */
  uint32_t       relax_sides;  /* DPPO_RELAX_HIGH | DPPO_RELAX_LOW: Relax-high, Relax-low, both */
  const void*    mu_logits;    /* bf16 [T, mu_ld]: the rollout policy's logits over the same   */
                               /* vocabulary (log-probs are logits too; any per-row shift is   */
                               /* immaterial).  DPPO_FULL_TV / DPPO_FULL_KL only, else ignored */
                               /* and may be NULL.  Must not overlap grad_logits.  r_t still   */
                               /* uses mu_logp                                                 */
  int64_t        mu_ld;        /* its row pitch in elements, mu_ld >= V                        */
  const float*   anchor_logp;  /* [T] or NULL.  log-prob of a_t under the policy the MASK is    */
                               /* anchored to when that is not the rollout policy: the trainer's*/
                               /* recomputed pi_theta' of the decoupled objectives.  With       */
                               /* DPPO_MASK_RATIO_CLIP this is MiniRL / MiniRL-TIS (App. C.1:   */
                               /* the clip on r' = pi / pi_theta'); with the divergence mask the*/
                               /* decoupled DPPO of Sec. 5.2 (D_t and the r' <> 1 test use it   */
                               /* where they use mu_logp otherwise; for the Top-K / full-       */
                               /* vocabulary variants pass that policy's top-K / logits too).   */
                               /* The weight min(r, C) and the loss keep r = pi / mu.           */
                               /* NULL: the mask is anchored to the rollout policy (DPPO, GRPO) */
  /* ---- outputs (fully overwritten) ---- */
  float*         loss;         /* [1]                                                          */
  float*         loss_tok;     /* [T] -M_t r_t A_t, unscaled; may be NULL                      */
  float*         divergence;   /* [T] D_t                                                      */
  uint8_t*       mask;         /* [T] M_t in {0, 1}                                            */
  void*          grad_logits;  /* bf16 [T, ld] (columns >= V untouched), round-to-nearest-even;*/
                               /* dppo_loss_fwd_bwd only; may be the same buffer as logits     */
                               /* (in place) but must not overlap it otherwise                 */
  float*         diagnostics;  /* [T, DPPO_NDIAG] per-token diagnostics (DPPO_DIAG_*), 16-byte  */
                               /* aligned; may be NULL.  Ignored rows get zeros               */
  /* ---- scratch ---- */
  void*          workspace;    /* dppo_workspace_bytes(T, V, K) bytes, 8-byte aligned; at      */
                               /* least DPPO_WORKSPACE_BYTES are required (DPPO_ERR_WORKSPACE  */
                               /* below that), and with less than dppo_workspace_bytes() the   */
                               /* long-row forward+backward kernel cannot hand its rows out at */
                               /* run time (about 2 % slower on 150k-entry rows).  Contents on */
                               /* entry are irrelevant; calls that overlap in time need        */
                               /* distinct workspaces                                          */
  size_t         workspace_bytes;
  uint32_t       flags;        /* DPPO_FLAG_*                                                  */
} dppo_args_t;

/* Bytes of device scratch for one call: DPPO_WORKSPACE_BYTES (per-workgroup partial sums of the
 * loss, row counters) + 8 T (one loss term per row, summed in a fixed order: the scalar loss is
 * the same whichever workgroup took which row). */
size_t dppo_workspace_bytes(int64_t T, int64_t V, int32_t K);

/* Forward only: loss, loss_tok, divergence, mask.  grad_logits is ignored.
 * T = 0 is valid and stores loss = 0.  (Sec. 4.3, Eq. dppo_obj; Sec. 4.4) */
dppo_status_t dppo_loss_fwd(const dppo_args_t* args, void* stream);

/* Forward and backward in one fused pass per row: the outputs of dppo_loss_fwd plus
 * grad_logits.  (Eq. dppo_obj for the loss, Eq. unified_grad with C = infinity for the
 * gradient.) */
dppo_status_t dppo_loss_fwd_bwd(const dppo_args_t* args, void* stream);

/* For callers that cannot allocate or pass device scratch (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): dppo_loss_fwd_bwd with the partial sums of the
 * loss kept in a static device array of DPPO_STATIC_SCRATCH_BYTES that the library itself holds on
 * every GPU it runs on, from load until the process ends.  `workspace` / `workspace_bytes` are
 * ignored (may be NULL / 0); inputs and outputs are passed as usual; the call allocates nothing
 * and clears nothing (every partial sum it reads it has written).  Limits and errors beyond
 * those of dppo_loss_fwd_bwd: T <= DPPO_STATIC_MAX_T, else DPPO_ERR_SHAPE; `stream` must belong
 * to the CURRENT device, else DPPO_ERR_LAUNCH; DPPO_ERR_WORKSPACE if the runtime yields no
 * address for the array.  All calls on one GPU share that GPU's array: calls that overlap in
 * time on one GPU (different streams, or a replaying graph beside eager calls) race on it and
 * return wrong losses; serialise them or use dppo_loss_fwd_bwd with distinct workspaces.  The
 * array's address is looked up on the first call on a device, or by dppo_static_init() -- call
 * that once per device, with the device current and outside any stream capture, if the first
 * call would otherwise fall inside a capture. */
#define DPPO_STATIC_SCRATCH_BYTES 65536
#define DPPO_STATIC_MAX_T (1 << 22)
dppo_status_t dppo_loss_fwd_bwd_static(const dppo_args_t* args, void* stream);
dppo_status_t dppo_static_init(void);

/* Static, NUL-terminated description of a status code. */
const char* dppo_status_str(dppo_status_t status);

/* DPPO_VERSION of the loaded library. */
int dppo_version(void);

/* sizeof(dppo_args_t) as the library was compiled: lets a foreign-language binding verify its
 * mirror of the struct. */
size_t dppo_args_size(void);

/* Name of the kernel path the last successful dppo_loss_* call on this thread chose:
 * "resident" (row held in registers between the two passes), "resident_long" (rows of 155657 ..
 * 262144 entries with the gradient: registers, LDS and a short tail read twice), "resident_multi"
 * (rows of 16392 .. 65536 entries with the gradient, many of them per call: groups of two to six
 * rows held in registers), "streaming" (row re-read),
 * "fullvocab" (the two-row kernel of the DPPO_FULL_* variants) or "fullvocab_resident" (their
 * backward, and the forward-only TV form, on long aligned rows: the trainer's row held in
 * registers, the rollout row streamed past it); "lmhead" after a dppo_lmhead_* call that went
 * through chunks of logits, "lmhead_fused" after a forward-only one that did not. */
const char* dppo_last_path(void);

/* ---- the same loss from the hidden states: the [T, V] logits never exist in full -------------
 * The full divergence and even the log-probabilities over a 150k vocabulary are what makes the
 * trust region expensive in memory (Sec. 4.4).  Here the caller hands over the final hidden
 * states h[T, d] and the lm_head weight W[V, d] (bf16, row-major, as an nn.Linear keeps it);
 * the library walks T in chunks of `chunk_rows` tokens:
 *     z_c = h_c W^T           bf16 logits of the chunk, fp32 accumulation, round to nearest even
 *     loss, D, M, and g_c = d loss / d z_c in place            (exactly dppo_loss_fwd_bwd on z_c)
 *     d loss / d h_c = g_c W  bf16, fp32 accumulation, W read as it lies
 *     d loss / d W  += g_c^T h_c   (optional) fp32, from g_c and h_c as they lie (no transposed copies)
 * so device memory holds one chunk of logits, not [T, V].  `loss` carries every per-token
 * input and output with the meaning it has in dppo_loss_fwd_bwd (its logits, ld, grad_logits,
 * mu_logits, workspace and flags fields are ignored); the DPPO_FULL_* variants are not
 * available here.  Needs V and d multiples of 64.  Outputs: those of `loss`, and grad_hidden. */
typedef struct {
  dppo_args_t    loss;          /* T, V, per-token inputs/outputs, variant, delta, loss_scale, ...  */
  const void*    hidden;        /* bf16 [T, ld_hidden], 16-byte aligned                            */
  int64_t        ld_hidden;     /* >= d, multiple of 8                                             */
  int64_t        d;             /* hidden size, multiple of 64                                     */
  const void*    weight;        /* bf16 [V, ld_weight]: lm_head weight, 16-byte aligned            */
  int64_t        ld_weight;     /* >= d, multiple of 8                                             */
  int64_t        chunk_rows;    /* tokens per chunk; <= 0: 8192.  The second and third products have  */
                                /* chunk_rows/256 x d/256 tiles: keep that at or above the number  */
                                /* of compute units (256)                                          */
  void*          grad_hidden;   /* bf16 [T, ld_grad_hidden]; dppo_lmhead_loss_fwd_bwd only         */
  int64_t        ld_grad_hidden;/* >= d                                                            */
  float*         grad_weight;   /* optional fp32 [V, ld_grad_weight], 16-byte aligned:             */
                                /* d loss / d W = g^T h summed over all T tokens; NULL = not wanted */
  int64_t        ld_grad_weight;/* >= d, multiple of 4                                             */
  int32_t        grad_weight_accumulate; /* 0: overwrite grad_weight; 1: add to what it holds (a   */
                                /* trainer accumulating micro-batches into an fp32 main gradient) */
  void*          workspace;     /* >= dppo_lmhead_workspace_bytes(...) bytes, 256-byte aligned:    */
                                /* loss partial sums and the chunk of logits                       */
  size_t         workspace_bytes;
} dppo_lmhead_args_t;

/* 64 KiB + min(chunk_rows, T) * V * 2 bytes (chunk_rows <= 0: the default); enough for either call. */
size_t dppo_lmhead_workspace_bytes(int64_t T, int64_t V, int64_t chunk_rows);

/* What dppo_lmhead_loss_fwd alone needs: 64 KiB + 8 T + min(chunk_rows, T) * (16 ceil(V / 256) +
 * 4 (K + 1)) bytes (each part rounded up to 256), K as the Top-K variants use it (0 for Binary). */
size_t dppo_lmhead_fwd_workspace_bytes(int64_t T, int64_t V, int32_t K, int64_t chunk_rows);

/* Forward only (loss, loss_tok, divergence, mask, diagnostics).  No logit is written to memory:
 * the product kernel itself reduces every 256 x 256 tile of bf16-rounded logits to per-row softmax
 * statistics (and picks the logits at the sampled and top-K ids out of the tile); a second small
 * kernel combines the tiles of a row and evaluates the loss.  The results are those of
 * dppo_loss_fwd on the bf16 logits.  (DPPO_FLAG_FORCE_STREAMING in loss.flags selects the general
 * route through a chunk of logits instead, for comparison; it needs the larger workspace.) */
dppo_status_t dppo_lmhead_loss_fwd(const dppo_lmhead_args_t* args, void* stream);

/* Forward and backward: also grad_hidden = d loss / d hidden and, if asked for, grad_weight. */
dppo_status_t dppo_lmhead_loss_fwd_bwd(const dppo_lmhead_args_t* args, void* stream);

/* sizeof(dppo_lmhead_args_t) as the library was compiled. */
size_t dppo_lmhead_args_size(void);

/* C[M, N] = A[M, K] * B[N, K]^T on the matrix cores: bf16 operands, both row-major with the
 * contraction index contiguous (activations [T, d] times an lm_head weight [V, d] transposed),
 * fp32 accumulation, C bf16 row-major rounded to nearest even.  The building block of the
 * logits-free path (the logits of a chunk of tokens, and the gradient with respect to the
 * hidden states from the gradient with respect to those logits).  K a multiple of 64; A and B
 * 16-byte aligned with lda, ldb multiples of 8 and below 2^22; C 2-byte aligned; buffers must not
 * overlap.  M = 0 or N = 0 is valid and does nothing. */
dppo_status_t dppo_gemm_nt(const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                           int64_t M, int64_t N, int64_t K, void* stream);

/* The same product with an fp32 result, C (+)= A B^T: C fp32 [M, ldc], 16-byte aligned with ldc a
 * multiple of 4; accumulate != 0 adds the product to what C holds.  (The weight gradient of the
 * path above sums its chunks this way.) */
dppo_status_t dppo_gemm_nt_f32(const void* A, int64_t lda, const void* B, int64_t ldb, float* C, int64_t ldc,
                               int64_t M, int64_t N, int64_t K, int accumulate, void* stream);

/* C[M, N] = A[M, K] * B[K, N]: A with the contraction index contiguous, B with the contraction
 * index as the ROW index (a gradient with respect to the logits [T, V] times the lm_head weight
 * [V, d] as it lies), bf16 in, fp32 accumulation, C bf16 rounded to nearest even.  K a multiple of
 * 64; A and B 16-byte aligned with lda >= K, ldb >= N multiples of 8 and below 2^22; C 2-byte
 * aligned, ldc >= N; buffers must not overlap.  Errors as for dppo_gemm_nt. */
dppo_status_t dppo_gemm_nn(const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                           int64_t M, int64_t N, int64_t K, void* stream);

/* C[M, N] (+)= A[K, M]^T * B[K, N]: both bf16 operands row-major with the contraction index as
 * the ROW index (what the gradient of a weight is: logit gradients [T, V] transposed times
 * activations [T, d]), read as they lie, fp32 accumulation, C fp32 [M, ldc].  Any K >= 1 (rows
 * past K count as zeros); A and B 16-byte aligned with lda >= M, ldb >= N multiples of 8 and
 * below 2^22; C 16-byte aligned with ldc >= N a multiple of 4; accumulate != 0 adds the product to
 * what C holds.  Device pointers, caller-owned; buffers must not overlap.  M = 0 or N = 0 is valid
 * and does nothing.  DPPO_ERR_SHAPE / _NULL / _ALIGN / _LAUNCH as for dppo_gemm_nt. */
dppo_status_t dppo_gemm_tn_f32(const void* A, int64_t lda, const void* B, int64_t ldb, float* C, int64_t ldc,
                               int64_t M, int64_t N, int64_t K, int accumulate, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DPPO_H */
