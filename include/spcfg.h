/*
 * spcfg.h - C ABI of the MI355X (gfx950) inside / inside-backward library for simple PCFGs.
 *
 * A simple PCFG (paper Sec. 2) has rules S -> A, A -> B C, T -> w with the binary rule probability
 * factored as pi(A -> B C) = L[A,B] * R[A,C].  A is a nonterminal (N of them); children B, C are
 * nonterminals or preterminals (P of them); M = N + P.  Column order of L and R: nonterminal children
 * in [0, N), preterminal children in [N, M).
 *
 * The library evaluates, for a batch of sentences, the inside recursion of Sec. 3.1
 *     beta_ij = sum_{i<k<j} (L beta_ik) * (R beta_kj)        (elementwise product, fencepost spans)
 * with base case beta_{i,i+1} = emission vector of token i, and Z = sum_A pi(S->A) beta_0n[A], in the
 * hardware-oriented form of Sec. 3.2 (all spans of one width per launch, the L and R projections as one
 * stacked matrix product, rescaling by the per-span maximum), and the reverse pass that Sec. 3.2
 * ("Recomputation") sketches: nothing per split point is kept from the forward pass.
 *
 * Conventions
 *   - "dev" pointers are device memory on the current HIP device, "host" pointers ordinary host memory.
 *   - Matrices are row-major and dense: L, R are [N x M]; log_emit is [B x n_max x P].
 *   - Every call only enqueues work on `hip_stream` (a hipStream_t, NULL = the default stream); results
 *     are valid once the caller has synchronised that stream.  Host arrays (lengths) are consumed before
 *     the call returns.  The library allocates no device memory; the caller owns every buffer.
 *   - Errors that can be seen on the host (null pointer, bad shape, bad length, workspace too small) are
 *     returned before anything is launched.  HIP runtime failures map to SPCFG_ERR_HIP.
 *   - Results are deterministic: no floating-point atomics are used.
 */
#ifndef SPCFG_H
#define SPCFG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  SPCFG_OK = 0,
  SPCFG_ERR_ARG = -1,         /* null pointer, bad struct_size, negative size                      */
  SPCFG_ERR_SHAPE = -2,       /* N, P, B or n_max outside the supported range or above capacity      */
  SPCFG_ERR_LENGTH = -3,      /* some lengths[b] < 2 or > n_max (a tree needs the rule S -> A, A -> B C) */
  SPCFG_ERR_WORKSPACE = -4,   /* workspace pointer misaligned or workspace_bytes too small            */
  SPCFG_ERR_UNSUPPORTED = -5, /* precision / flag combination not implemented                         */
  SPCFG_ERR_HIP = -6,         /* a HIP runtime call failed (see spcfg_last_hip_error)                 */
  SPCFG_ERR_STATIC_CAPACITY = -7 /* spcfg_inside_static: the batch needs more than SPCFG_STATIC_SCRATCH_BYTES  */
};

enum { SPCFG_PRECISION_FP32 = 0, SPCFG_PRECISION_BF16 = 1 };

enum {
  SPCFG_FLAG_ACCUMULATE_GRADS = 1u, /* add into grad_L / grad_R / grad_log_root instead of overwriting */
  /* One grammar per sentence (the dynamic program of the compound variant, App. A: rule probabilities that
     depend on a per-sentence latent vector).  log_root is then [B x N], L and R are [B x N x M], and
     grad_log_root, grad_L, grad_R have the same per-sentence shapes (no sum over the batch).  The projections
     become grouped products: each sentence's spans meet that sentence's [L;R] panel.  With
     SPCFG_PRECISION_BF16 the forward projections then read fp32 operands (so that log Z keeps its bound), the
     reverse projections bf16 ones, and the per-sentence rule gradients are reduced with fp32 operands. */
  SPCFG_FLAG_PER_SENTENCE_GRAMMAR = 2u,
  /* SPCFG_PRECISION_FP32 forms its matrix products from bf16 matrix instructions by default: every fp32
     operand is cut exactly into three bf16 pieces and six piece products are accumulated in fp32, which keeps
     the accuracy of an fp32 product (the dropped terms are below 2^-23 of it) at a fraction of the cost of
     fp32 matrix instructions.  This flag selects fp32 matrix instructions instead.  It has no effect on products
     whose operands are bf16 (SPCFG_PRECISION_BF16). */
  SPCFG_FLAG_FP32_MFMA = 4u,
  /* SPCFG_PRECISION_BF16 with a shared grammar forms its forward projection products -- the ones log Z depends on --
     from operands cut into two bf16 pieces (hi + lo, three piece products, operands good to 2^-17), so that log Z
     stays within about 1e-3 of exact arithmetic whatever the grammar and the sentence length.  This flag rounds those
     operands to a single bf16 instead, as the reverse and rule-gradient products always do: a third of the matrix
     work in the forward products (the Scaled configuration takes 16 % less time), but roundings of 2^-9 per projection
     then add up along a tree: measured up to 0.07 absolute in log Z on small peaked grammars with sentences of
     60-100 words, 0.6e-3 to 1.5e-3 on large unpeaked ones at n = 40.  With one grammar per sentence the flag replaces
     the fp32 operands of the forward products by single bf16 ones.  No effect with SPCFG_PRECISION_FP32. */
  SPCFG_FLAG_BF16_SINGLE_FORWARD = 8u
};

/* Plain-old-data configuration; set struct_size = sizeof(spcfg_config). */
typedef struct {
  uint32_t struct_size;
  int32_t N;         /* number of nonterminals, >= 1                                              */
  int32_t P;         /* number of preterminals, >= 1                                              */
  int32_t max_B;     /* capacity: largest batch the workspace is sized for                        */
  int32_t max_n;     /* capacity: largest sentence length the workspace is sized for              */
  int32_t precision; /* SPCFG_PRECISION_FP32: fp32 operands on the matrix cores, fp32 accumulate;
                        SPCFG_PRECISION_BF16: the operands of the projection and rule-gradient
                        products are bf16 (two bf16 pieces per value in the forward projections of a
                        shared grammar, see SPCFG_FLAG_BF16_SINGLE_FORWARD), fp32 accumulate; everything
                        else stays fp32.  Gradients carry the single-bf16 roundings of the reverse
                        products: relative L2 error 1e-4 .. 1e-2 per tensor on large unpeaked grammars,
                        up to a few 1e-2 on small peaked ones */
  uint32_t flags;    /* SPCFG_FLAG_*                                                              */
} spcfg_config;

/* Upper bound of the workspace needed for any batch with B <= max_B, every length <= max_n. */
int spcfg_workspace_bytes(const spcfg_config* cfg, size_t* out_bytes);

/* Exact workspace need of one batch (host `lengths`); never more than spcfg_workspace_bytes. */
int spcfg_workspace_bytes_for(const spcfg_config* cfg, const int32_t* lengths, int32_t B, int32_t n_max,
                              size_t* out_bytes);

/*
 * Inside pass (Sec. 3.1 recursion, Sec. 3.2 schedule): logZ[b] = log Z of sentence b.
 *   log_root  dev [N]             log pi(S -> A); any log-weights, -inf allowed
 *   L, R      dev [N x M]         non-negative weights (probability space), M = N + P
 *   log_emit  dev [B x n_max x P] log pi(T -> w_{b,i}); positions i >= lengths[b] are never read
 *   lengths   host [B]            2 <= lengths[b] <= n_max <= max_n
 *   logZ      dev [B]             out; -inf for a sentence the grammar cannot derive
 *   workspace dev, 256-byte aligned, >= spcfg_workspace_bytes_for(...) bytes.  After the call it holds
 *             the chart (scaled inside vectors and their L/R projections for every span) that
 *             spcfg_inside_backward needs; it must stay untouched until that call has run.
 */
int spcfg_inside(const spcfg_config* cfg, const float* log_root, const float* L, const float* R,
                 const float* log_emit, const int32_t* lengths, int32_t B, int32_t n_max, float* logZ,
                 void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Reverse pass (Sec. 3.2 "Recomputation"; chain rule through the stacked projection): gradients of
 * sum_b grad_logZ[b] * logZ[b].  Must follow spcfg_inside on the same inputs, workspace and stream order.
 *   grad_logZ      dev [B] or NULL (= all ones)
 *   grad_L, grad_R dev [N x M]  d/dL[A,B], d/dR[A,C] in probability space, summed over the batch;
 *                               L*grad_L and R*grad_R are expected rule counts
 *   grad_log_root  dev [N]      summed over the batch; with grad_logZ = 1 the root posteriors
 *   grad_log_emit  dev [B x n_max x P]  per sentence (preterminal posteriors); 0 at padded positions
 * Sentences with Z = 0 contribute nothing.  Gradients are overwritten unless SPCFG_FLAG_ACCUMULATE_GRADS
 * (which applies to grad_L, grad_R, grad_log_root; grad_log_emit is always overwritten).
 */
int spcfg_inside_backward(const spcfg_config* cfg, const float* log_root, const float* L, const float* R,
                          const float* log_emit, const int32_t* lengths, int32_t B, int32_t n_max,
                          const float* grad_logZ, float* grad_L, float* grad_R, float* grad_log_root,
                          float* grad_log_emit, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * spcfg_inside for callers that cannot allocate device memory or pass a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same kernels, with the whole workspace (chart,
 * exponents, packed panels, partial tiles and arrival counters of the projection products) in a static device array
 * of SPCFG_STATIC_SCRATCH_BYTES that lives in the library's code object.  Nothing is allocated or freed, by this
 * call or by anything it calls.  Arguments as for spcfg_inside.
 *   - A batch whose workspace need exceeds the array (see spcfg_workspace_bytes_for; the static layout keeps 56 MiB
 *     less partial-tile scratch than that figure) is refused with SPCFG_ERR_STATIC_CAPACITY before anything is
 *     launched.  Small grammars fit (N = P = 512 with a few hundred words per batch), the headline one does not.
 *   - Every GPU holds its own copy of the array until the process ends; the address is looked up on the first call
 *     on a device (that device current).  All calls on one GPU share it and it keeps the last call's contents
 *     (whatever has to start at zero is cleared by the call's first kernels): calls that overlap on one GPU, on
 *     different streams or from different threads, race.  No backward call can follow: the chart is not the caller's.
 */
#define SPCFG_STATIC_SCRATCH_BYTES (64u << 20)
int spcfg_inside_static(const spcfg_config* cfg, const float* log_root, const float* L, const float* R,
                        const float* log_emit, const int32_t* lengths, int32_t B, int32_t n_max, float* logZ,
                        void* hip_stream);

/* spcfg_inside followed by spcfg_inside_backward on the same stream (one call for the fwd+bwd step). */
int spcfg_inside_forward_backward(const spcfg_config* cfg, const float* log_root, const float* L,
                                  const float* R, const float* log_emit, const int32_t* lengths, int32_t B,
                                  int32_t n_max, const float* grad_logZ, float* logZ, float* grad_L,
                                  float* grad_R, float* grad_log_root, float* grad_log_emit, void* workspace,
                                  size_t workspace_bytes, void* hip_stream);

/* Static, never-NULL description of an error code. */
const char* spcfg_strerror(int code);

/* Text of the last HIP runtime error seen by this thread's calls ("" if none). */
const char* spcfg_last_hip_error(void);

/*
 * Per-kernel-class timing.  While enabled, every kernel launch carries a pair of HIP events bound to the start
 * and the end of that kernel on the caller's stream; a class's time is the sum of its kernels' durations
 * (this perturbs the schedule slightly, so whole-step timing should be taken with profiling disabled).
 * spcfg_profile_read synchronises the recorded events, then fills, for class c in [0, SPCFG_PROF_CLASSES):
 *   ms[c]      total device time of the class since spcfg_profile_enable(1)
 *   launches[c] number of launches
 *   work[c]    algorithmic work enqueued: flop for the GEMM classes, bytes for the others
 * and resets the counters.  Arrays must hold SPCFG_PROF_CLASSES entries.  The counters are the library's only state:
 * process-wide and guarded by a mutex; launches of all threads made while profiling is enabled add up.
 */
enum {
  SPCFG_PROF_SETUP = 0,      /* span plan, weight packing, leaf preparation                            */
  SPCFG_PROF_GEMM_FWD = 1,   /* stacked [L;R] projection GEMMs of the inside pass                      */
  SPCFG_PROF_SPLIT_FWD = 2,  /* split-point reduction of the inside pass                               */
  SPCFG_PROF_ROOT = 3,       /* root reductions (forward and backward)                                 */
  SPCFG_PROF_SPLIT_BWD = 4,  /* gather of parent adjoints times sibling projections                    */
  SPCFG_PROF_GEMM_BWD = 5,   /* projection of adjoints back through [L;R]                              */
  SPCFG_PROF_GEMM_GRAD = 6,  /* rule-gradient GEMMs (reduction over all spans)                         */
  SPCFG_PROF_CLASSES = 7
};
int spcfg_profile_enable(int on);
int spcfg_profile_read(double* ms, int64_t* launches, double* work);
const char* spcfg_profile_class_name(int cls);

/*
 * Rule-probability front-end (the softmaxes that end the neural parameterisation, App. A) and its backward.
 * The scores ("logits") are what the paper's networks produce; the outputs are what spcfg_inside consumes.
 *   root_logits dev [N], L_logits / R_logits dev [N x M], emis_logits dev [P x V]  (V = vocabulary size)
 *   tokens      dev [B x n_max] int32 token ids in [0, V); entries at i >= lengths[b] are ignored
 *   lengths     host [B], 0 <= lengths[b] <= n_max
 * spcfg_rules_forward writes
 *   log_root = log_softmax(root_logits) [N];  L = softmax rows of L_logits, R likewise [N x M];
 *   log_emit[b, i, T] = log_softmax(emis_logits[T, :])[tokens[b, i]]  [B x n_max x P], 0 at padded positions
 *                       (NaN if a token id is out of range);
 *   emis_lse[T] = logsumexp(emis_logits[T, :]) [P], kept for the backward call.
 * The P x V emission table is the dominant cost here at scale (paper, Limitations): it is read once for
 * the row reductions and gathered once per token.
 */
int spcfg_rules_forward(int32_t N, int32_t P, int32_t V, const float* root_logits, const float* L_logits,
                        const float* R_logits, const float* emis_logits, const int32_t* tokens, const int32_t* lengths,
                        int32_t B, int32_t n_max, float* log_root, float* L, float* R, float* log_emit, float* emis_lse,
                        void* hip_stream);

/*
 * Backward of spcfg_rules_forward: gradients w.r.t. the four logit arrays given gradients w.r.t. its outputs
 * (e.g. those written by spcfg_inside_backward).  log_root, L, R, emis_lse are the forward outputs.
 *   grad_root_logits dev [N], grad_L_logits / grad_R_logits dev [N x M], grad_emis_logits dev [P x V]: overwritten
 *   scratch          dev [32 x P] floats of scratch
 * Deterministic: equal tokens are accumulated in a fixed order, no floating-point atomics.
 */
int spcfg_rules_backward(int32_t N, int32_t P, int32_t V, const float* log_root, const float* L, const float* R,
                         const float* emis_logits, const float* emis_lse, const int32_t* tokens,
                         const int32_t* lengths, int32_t B, int32_t n_max, const float* grad_log_root,
                         const float* grad_L, const float* grad_R, const float* grad_log_emit, float* grad_root_logits,
                         float* grad_L_logits, float* grad_R_logits, float* grad_emis_logits, float* scratch,
                         void* hip_stream);

/*
 * Span posteriors (the quantity the reverse pass of the inside algorithm yields, Sec. 3.2: back-propagation
 * through the inside recursion is the outside pass, and beta * d logZ / d beta is the span marginal).
 * Reads the workspace left by spcfg_inside + spcfg_inside_backward (or the fused call) for the same cfg,
 * lengths, B, n_max; the workspace is not modified.
 *   span_post  dev [B x n_max x n_max], entry ((b * n_max + i) * n_max + (j - 1)) for the fencepost span
 *              (i, j), 0 <= i < j <= lengths[b]:  sum_A P(A spans (i,j) | sentence b) * grad_logZ[b].
 *              Width-1 entries carry the root span's value (both are in every tree); all other entries 0.
 *   span_label dev, same shape, or NULL: the nonterminal with the largest marginal on spans of width >= 2
 *              (smallest index on ties), -1 elsewhere or where the posterior is 0.
 */
int spcfg_span_marginals(const spcfg_config* cfg, const int32_t* lengths, int32_t B, int32_t n_max,
                         const void* workspace, size_t workspace_bytes, float* span_post, int32_t* span_label,
                         void* hip_stream);

/*
 * Minimum-Bayes-risk tree (the parse used to score a grammar as an unsupervised parser, Sec. 4 "Evaluation"):
 * the binary bracketing of each sentence that maximises the sum of span_post over its spans of width >= 2,
 * by CKY over split points; the smallest split point wins ties.
 *   span_post  dev [B x n_max x n_max], layout as written by spcfg_span_marginals (any non-negative scores; with
 *              -inf or NaN scores the result is still a valid bracketing - a span whose candidates are all -inf
 *              or NaN takes its smallest split point - and tree_score is -inf or NaN)
 *   lengths    host [B], 2 <= lengths[b] <= n_max <= 1024;  B <= 960
 *   tree_spans dev [B x (n_max - 1) x 2] int32: the lengths[b] - 1 spans (i, j) of width >= 2 in pre-order
 *              (parent, left subtree, right subtree), then -1 padding
 *   tree_score dev [B]: the maximised sum
 *   scratch    dev, 16-byte aligned, >= spcfg_mbr_decode_scratch_bytes(B, n_max) bytes
 */
int spcfg_mbr_decode_scratch_bytes(int32_t B, int32_t n_max, size_t* out_bytes);
int spcfg_mbr_decode(const float* span_post, const int32_t* lengths, int32_t B, int32_t n_max, int32_t* tree_spans,
                     float* tree_score, void* scratch, size_t scratch_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SPCFG_H */
