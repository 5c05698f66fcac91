/*
 * del.h - C ABI of the MI355X (gfx950) library for the greedy self-speculative
 * decode round with DEL (Dynamic Exit Layer, arXiv 2504.05598).
 *
 * One context = one Llama-style decoder resident on one GPU, one KV cache,
 * one sequence (batch 1).  The call order is
 *     del_create -> del_load_weights (until every tensor is loaded)
 *                -> del_prefill -> del_round* [-> del_prefill -> ...]
 * Every entry point returns a del_status, never throws and never aborts.
 * Unless a parameter says "device", pointers are HOST pointers owned by the
 * caller; outputs are caller-allocated.  A context is not thread-safe.  All GPU
 * work of a context runs on the stream given to del_create and every call has
 * completed its GPU work when it returns.
 *
 * Layer numbering follows the paper (Section 2): layers 1..L, h^0 is the
 * embedding of the input token, h^l the output of layer l.  Exit layer E is
 * the number of layers the draft runs.
 */
#ifndef DEL_H
#define DEL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct del_ctx del_ctx; /* opaque; owned by the library */

typedef enum {
  DEL_OK = 0,
  DEL_E_ARG = 1,      /* null pointer, value out of range                      */
  DEL_E_STATE = 2,    /* call out of order (e.g. round before prefill)         */
  DEL_E_CAPACITY = 3, /* KV cache would exceed max_context; state unchanged    */
  DEL_E_SHAPE = 4,    /* tensor shape does not match the configuration         */
  DEL_E_DEVICE = 5,   /* a HIP call failed; del_last_error_text has the detail */
  DEL_E_NOMEM = 6     /* device or host allocation failed                      */
} del_status;

enum { DEL_DTYPE_FP32 = 0, DEL_DTYPE_BF16 = 1 };
enum { DEL_MEM_HOST = 0, DEL_MEM_DEVICE = 1 };

/* Model shape and DEL hyper-parameters. */
typedef struct {
  int32_t n_layers;        /* L                                                     */
  int32_t d_model;
  int32_t n_q_heads;
  int32_t n_kv_heads;      /* divides n_q_heads; q head j reads kv head j/(nq/nkv)  */
  int32_t head_dim;        /* multiple of 16; n_q_heads*head_dim need not = d_model */
  int32_t d_ffn;           /* multiple of 8                                         */
  int32_t vocab;
  float rope_theta;
  float rms_eps;
  int32_t tied_embeddings; /* 1: the LM head is the embedding matrix                */
  int32_t weight_dtype;    /* DEL_DTYPE_*; matrices only, norm gains are fp32.
                              The KV cache is stored in the same type.              */
  int32_t max_context;     /* KV rows per layer; >= prompt + generated + d_max + 1  */
  int32_t d_max;           /* cap on the speculation length gamma (Section 4.3)     */
  int32_t prefill_window;  /* prompt positions that seed the statistics (App. B.2)  */
  double omega;            /* decay of the weighted sum S (Section 4.2, App. B.2)   */
  int32_t use_mfma;        /* 1: multi-row GEMMs on the matrix cores (bf16 weights);
                              0: plain vector-ALU kernels everywhere                */
} del_config;

typedef enum {
  DEL_T_EMBED = 0, DEL_T_LM_HEAD = 1, DEL_T_FINAL_NORM = 2,
  DEL_T_ATTN_NORM = 3, DEL_T_WQ = 4, DEL_T_WK = 5, DEL_T_WV = 6, DEL_T_WO = 7,
  DEL_T_FFN_NORM = 8, DEL_T_WG = 9, DEL_T_WU = 10, DEL_T_WD = 11
} del_tensor_kind;

/* One weight tensor, row-major [rows, cols] = [out_features, in_features]
 * (norm gains: rows = 1).  Matrices are in cfg.weight_dtype, gains in fp32. */
typedef struct {
  int32_t layer;    /* 0..L-1; -1 for EMBED / LM_HEAD / FINAL_NORM            */
  int32_t kind;     /* del_tensor_kind                                        */
  int32_t location; /* DEL_MEM_HOST or DEL_MEM_DEVICE: where `data` lives     */
  int32_t reserved;
  const void* data; /* caller keeps ownership; copied before the call returns */
  int64_t rows, cols;
} del_tensor;

/* Create a context: allocates weights, KV cache and work buffers on the
 * current HIP device.  `hip_stream` is a hipStream_t (NULL = default stream). */
del_status del_create(const del_config* cfg, void* hip_stream, del_ctx** out);
void del_destroy(del_ctx* ctx);

/* Copy `n` tensors into the context, re-tiling them into the layout the
 * kernels stream (the decoder of Section 2, "Auto-regressive decoding"; the
 * paper treats Transformer_l as a black box, the block is the pre-norm Llama
 * block).  May be called repeatedly with subsets (one layer at a time for the
 * largest shapes).  With tied embeddings LM_HEAD must not be loaded.
 * Errors: DEL_E_SHAPE on a shape mismatch, DEL_E_ARG on bad layer/kind/pointer. */
del_status del_load_weights(del_ctx* ctx, const del_tensor* tensors, int32_t n);

/* Prefill (Section 4.3; Algorithm 1, initialisation; Appendix B.2): resets the KV
 * cache and the statistics, runs all L layers over the `n_prompt` prompt tokens,
 * seeds the per-layer acceptance statistics from the last
 * min(prefill_window, n_prompt) positions (every layer's shadow token against
 * layer L's), returns the first generated token and the first (E, gamma).
 * Errors: DEL_E_STATE before all weights are loaded; DEL_E_CAPACITY if
 * n_prompt + 1 > max_context; DEL_E_ARG for ids outside [0, vocab). */
del_status del_prefill(del_ctx* ctx, const int32_t* prompt, int32_t n_prompt,
                       int32_t* first_token, int32_t* next_E, int32_t* next_gamma);

/* One greedy self-speculative round (Section 2, "Early-exit self-speculative
 * decoding"; Algorithm 1, loop body without the confidence break):
 *   draft   gamma tokens with layers 1..E + final norm + LM head + arg-max;
 *   verify  the gamma+1 positions through layers E+1..L, reusing the exit-layer
 *           hidden states and the KV cache, accept the longest matching prefix;
 *   DEL     shadow tokens of every layer for the gamma+1 positions, u_r, c_r^l,
 *           decayed sums, alpha_l, TPL arg-max (Sections 4.1-4.3, Eq. 1-2).
 * 1 <= E <= L, 0 <= gamma <= d_max.  out_tokens has room for gamma+1 ids;
 * *n_out in [1, gamma+1] = accepted drafts + 1 token of the target model.
 * The selected (E, gamma) for the next round is read with del_layer_stats.
 * Errors: DEL_E_STATE before prefill, DEL_E_ARG, DEL_E_CAPACITY (state unchanged). */
del_status del_round(del_ctx* ctx, int32_t E, int32_t gamma, int32_t* out_tokens, int32_t* n_out);

/* The same round with dynamic draft-exiting (Section 4.4, Eq. 3; Algorithm 1, draft loop):
 * drafting runs for up to d_cap <= d_max steps and stops, before appending it, at the first token
 * whose confidence (soft-max probability of the drafted token) is below `tau` >= 0 - normally the
 * tau of layer E from del_layer_stats.  The hidden state of the stopping step is the round's last
 * row, so no extra pass over the first E layers is needed.  out_tokens has room for d_cap+1 ids.
 * *gamma_used = tokens drafted, *stopped_early = 1 if the loop stopped on low confidence (either
 * may be NULL).  The host decides after every draft step: the step's head kernel writes one 8-byte word
 * (sequence number, confidence) into pinned host memory, which the host polls (bounded; past 20 ms it
 * falls back to waiting for the stream), so a draft step costs one host round trip. */
del_status del_round_dynamic(del_ctx* ctx, int32_t E, double tau, int32_t d_cap, int32_t* out_tokens,
                             int32_t* n_out, int32_t* gamma_used, int32_t* stopped_early);

/* Per-layer statistics (Section 4.2; Eq. 2).  Arrays are caller-allocated and
 * indexed by layer number 0..L (entry 0 unused).  Any array pointer may be NULL. */
typedef struct {
  int32_t n_layers, rounds;  /* rounds since prefill                               */
  int32_t next_E, next_gamma;/* arg-max of TPL after the last update               */
  int32_t last_E, last_gamma, last_u, last_n; /* last round: u_r and n_r = u_r + 1 */
  double S_n;                /* decayed sum of valid-position counts               */
  double* S_c;               /* [L+1] decayed sums of matched counts               */
  double* alpha;             /* [L+1] S_c[l] / S_n                                 */
  int32_t* last_c;           /* [L+1] c_r^l of the last round (or of the prefill)  */
  int32_t* last_shadow;      /* [(L+1)*(d_max+1)] shadow ids, row-major by layer;
                                row l, entries 0..last_gamma (prefill: not filled) */
  int32_t* last_draft;       /* [d_max] drafted ids of the last round              */
  /* dynamic draft-exiting (Section 4.4): decayed confidence sums over matched / mismatched
   * shadow tokens and the threshold tau_l of Eq. 3 (a ratio with a zero denominator counts
   * as 0; mismatches = valid positions - matches)                                        */
  double* S_tcs;             /* [L+1]                                              */
  double* S_fcs;             /* [L+1]                                              */
  double* tau;               /* [L+1]                                              */
  float* last_conf;          /* [(L+1)*(d_max+1)] confidence of each shadow token, like last_shadow */
  float* last_draft_conf;    /* [d_max+1] confidence of each draft step taken (incl. a stopping one) */
  int32_t last_stopped;      /* 1 if the last round's draft loop stopped on low confidence */
} del_stats;
del_status del_layer_stats(const del_ctx* ctx, del_stats* out);
/* Import S_n and S_c, and S_tcs / S_fcs when both are non-NULL (resume, or re-synchronise a
 * test harness); recomputes alpha, tau and the next (E, gamma).  Nothing else is read.
 * Errors: DEL_E_ARG for S_n <= 0 or a negative sum; the statistics are then unchanged. */
del_status del_set_layer_stats(del_ctx* ctx, const del_stats* in);

/* Wall time of the segments of the last round, from HIP events on the stream. */
del_status del_last_timings(const del_ctx* ctx, float* draft_ms, float* verify_ms, float* shadow_ms);

/* Test hooks.  Hidden state of layer `layer` (0..L), row `row` of the last
 * round (0..gamma) or of the last prefill chunk, as d_model floats. */
del_status del_debug_hidden(const del_ctx* ctx, int32_t layer, int32_t row, float* dst);
/* Logits (vocab floats) of the LM head applied, after the final norm, to that row. */
del_status del_debug_logits(del_ctx* ctx, int32_t layer, int32_t row, float* dst);
/* Rows of the hidden-state buffer the last pass filled: after del_prefill the last prompt position is row
 * rows - 1 (for del_debug_hidden / del_debug_logits). */
del_status del_debug_last_rows(const del_ctx* ctx, int32_t* rows);
/* Current KV length T and the pending input token. */
del_status del_debug_state(const del_ctx* ctx, int32_t* kv_len, int32_t* pending_token);
/* Replace the pending input token (the token the next round starts from).  A lock-step
 * test harness uses it after re-prefilling on a context whose last prediction is a near-tie. */
del_status del_debug_set_pending(del_ctx* ctx, int32_t token);

/* Measurement hooks: a pure streaming read of `bytes` of the weight arena with
 * the GEMV kernels' access pattern (sets the achievable-bandwidth ceiling), and
 * the time of the last such call in ms. */
del_status del_bench_stream_read(del_ctx* ctx, int64_t bytes, int32_t iters, float* ms_per_iter);
/* The draft path's one-row GEMV (Section 4.1: a draft step streams E layers of weights for one row)
 * with parts of it switched off, timed over `iters` back-to-back launches on an n_blocks x k_tiles
 * tile matrix taken from the weight arena (consecutive launches read different parts of it): where a
 * launch spends its time beyond the weight stream.  parts: bit 0 = input row and gain staged through
 * LDS, bit 1 = bf16 decode + fp32 FMA, bit 2 = cross-wave reduction + RMS scale + residual store;
 * 0 = the tile loads alone in the GEMV's geometry.  waves per 16-row block: 4, 8 or 16; k_tiles <= 480.
 * Results of the arithmetic are discarded.  us_per_launch: host pointer.  DEL_E_ARG for arguments out
 * of range, DEL_E_CAPACITY if the matrix is larger than the arena. */
del_status del_bench_gemv_parts(del_ctx* ctx, int32_t n_blocks, int32_t k_tiles, int32_t waves, int32_t parts,
                                int32_t iters, float* us_per_launch);
/* Issue rate of the matrix instructions the shadow-head GEMM (Section 4.2) and the prefill GEMMs are built
 * from: 256 work-groups of 4 waves (one wave per SIMD) each run `iters` rounds of n_acc independent
 * accumulations with no memory traffic.  shape 0: v_mfma_f32_16x16x32_bf16, n_acc 2, 4, 8 or 16; shape 1:
 * v_mfma_f32_32x32x16_bf16, n_acc 1, 2 or 4.  ns_per_instruction (host pointer): nanoseconds per instruction
 * and SIMD; flops per instruction: 16384 (shape 0), 32768 (shape 1).  DEL_E_ARG otherwise. */
del_status del_bench_mfma_rate(del_ctx* ctx, int32_t shape, int32_t n_acc, int32_t iters, float* ns_per_instruction);
/* A plain device-to-device copy kernel of `bytes` (reads and writes that many bytes of a
 * temporary buffer): the known-size kernel the profiler's HBM byte counters are scaled by. */
del_status del_bench_stream_copy(del_ctx* ctx, int64_t bytes, int32_t iters, float* ms_per_iter);

/* Per-kernel timing for the roofline report.  While enabled, every GEMM launch of del_round
 * carries a pair of HIP events that receive the kernel's own start and stop timestamps
 * (hipExtLaunchKernel); per kernel class the launch count and the summed duration are
 * accumulated (throughput is still measured with profiling off).  A class is one kernel instantiation:
 * flavour (0 vector-ALU GEMV/GEMM, 1 matrix-core skinny GEMM, 2 shadow-head GEMM, 3 wide prefill GEMM, 4 and 5: the forms of 0 (one row)
 * and 1 that take several row blocks per work-group, 6: the register-blocked form of 2), epilogue (0 store, 1 residual, 2 qkv+rotary,
 * 3 swiglu, 4 argmax), rows m, matrix size.  weight_bytes is what one launch of the class streams. */
typedef struct {
  int32_t flavour, epilogue, rows, launches;
  double total_ms;
  int64_t weight_bytes;    /* tile bytes streamed per launch (part of what makes a class) */
} del_prof_entry;
del_status del_profile_enable(del_ctx* ctx, int32_t on);   /* also clears the counters */
del_status del_profile_read(const del_ctx* ctx, del_prof_entry* out, int32_t cap, int32_t* n);

/* Speculative sampling (Section 2, "Speculative decoding"; temperature and top_p of the inference
 * setup in the appendix).  A logits row is turned into soft-max(logits / temperature) restricted to
 * the nucleus of mass top_p (tokens by falling logit, lower id first among equals; the shortest
 * leading run whose mass reaches top_p) and renormalised; a uniform number r in [0, 1) draws the
 * first token, in id order, whose cumulative probability exceeds r.
 *
 * del_sample_first: only directly after del_prefill.  Replaces the greedy pending token by one drawn
 *   with `r` from the target's distribution at the last prompt position; *token receives it.
 * del_round_sample: one round like del_round, but the gamma drafts are drawn from the exit layer's
 *   distributions, a draft x is accepted when r * q(x) < p(x) (probability min(1, p(x)/q(x))), the
 *   first rejected position is redrawn from max(0, p - q) renormalised, and after gamma acceptances
 *   one more token is drawn from p.  uniforms (host, 2*gamma+1 numbers in [0, 1)): gamma for the
 *   drafts, gamma for the acceptances, one for the last token.  out_tokens (host, >= gamma+1) receives
 *   the accepted drafts and the last token, *n_out their number.  Shadow tokens stay greedy at every
 *   layer and the statistics count them over rows 0..u with u the number of accepted drafts.
 *   temperature > 0, 0 < top_p <= 1, else DEL_E_ARG; otherwise the errors of del_round.
 * del_round_sample_dynamic: del_round_sample with dynamic draft-exiting on top (Section 4.4): d_cap caps
 *   the draft length and drafting stops, before a token is drawn, at the first step whose confidence
 *   (temperature-1 soft-max probability of the exit layer's greedy token) is below tau >= 0.  uniforms has
 *   2*d_cap+1 numbers and every draw keeps its place: draft i uses uniforms[i], acceptance i
 *   uniforms[d_cap+i], the last token uniforms[2*d_cap].  *gamma_used / *stopped_early as in
 *   del_round_dynamic.
 * del_debug_spec_sample: the same sampling arithmetic on logits the caller supplies (host,
 *   q_logits [gamma][vocab], p_logits [gamma+1][vocab], row-major); no model, no state change.
 *   drafts_out (host, gamma ints; may be NULL when gamma == 0), *u, *last_token. */
del_status del_sample_first(del_ctx* ctx, double temperature, double top_p, float r, int32_t* token);
del_status del_round_sample(del_ctx* ctx, int32_t E, int32_t gamma, double temperature, double top_p,
                            const float* uniforms, int32_t* out_tokens, int32_t* n_out);
del_status del_round_sample_dynamic(del_ctx* ctx, int32_t E, double tau, int32_t d_cap, double temperature,
                                    double top_p, const float* uniforms, int32_t* out_tokens, int32_t* n_out,
                                    int32_t* gamma_used, int32_t* stopped_early);
del_status del_debug_spec_sample(del_ctx* ctx, const float* q_logits, const float* p_logits, int32_t gamma,
                                 double temperature, double top_p, const float* uniforms, int32_t* drafts_out,
                                 int32_t* u, int32_t* last_token);

/* For callers that cannot allocate device memory or have the library do so: code that is being captured
 * into a HIP graph, tight serving loops, harnesses that forbid hipMalloc.  The sampling arithmetic of
 * del_debug_spec_sample on logits that are already in DEVICE memory, with no context: every intermediate
 * (fixed-point weights, per-row records, counters) lives in one fixed device array of the library
 * (about 4.5 MB per GPU, held until the process ends).  The call allocates nothing, copies nothing to or
 * from the host and does not wait: it queues four kernels on `hip_stream` (NULL = default stream).
 *   q_logits  device, [gamma][ld_logits] floats (may be NULL when gamma == 0); p_logits device,
 *             [gamma+1][ld_logits]; both 16-byte aligned, ld_logits a multiple of 4 and >= vocab
 *   uniforms  device, 2*gamma+1 floats in [0, 1): drafts, acceptances, last token (not checked)
 *   out       device, 3+gamma ints: out[0] = u (accepted drafts), out[1] = u + 1, out[2] = the last
 *             token, out[3..3+gamma) = the drafted tokens; valid once the stream has passed the call
 * Limits: vocab <= 32768 and gamma <= 8, else DEL_E_CAPACITY; DEL_E_ARG for bad pointers, alignment,
 * temperature <= 0 or top_p outside (0, 1].  All calls on one GPU share the one array: calls whose
 * kernels may overlap on that GPU (different streams or threads of one process) race. */
del_status del_spec_sample_static(const float* q_logits, const float* p_logits, int64_t ld_logits, int32_t vocab,
                                  int32_t gamma, double temperature, double top_p, const float* uniforms,
                                  int32_t* out, void* hip_stream);

/* Host-only helpers (no context, no device): the policy arithmetic the library applies after
 * every round, exposed so that it can be checked on its own.
 * del_policy_step: one update of the running sums (Section 4.2: S <- omega*S + a for c^l, n, and
 * Section 4.4 for tcs^l, fcs^l; arrays indexed by layer number 0..L, entry 0 unused; tcs/fcs and
 * their sums may be NULL), then alpha_l (Eq. 2), tau_l (Eq. 3; NULL to skip) and the arg-max of
 * TPL(l, d) over l in [1, L), d in [0, d_max] (Eq. 1, Section 4.3; first maximum, l then d ascending). */
del_status del_policy_step(int32_t n_layers, int32_t d_max, double omega, const int32_t* c, int32_t n,
                           const double* tcs, const double* fcs, double* S_c, double* S_n, double* S_tcs,
                           double* S_fcs, double* alpha, double* tau, int32_t* next_E, int32_t* next_gamma);

const char* del_strerror(del_status s);
const char* del_last_error_text(const del_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* DEL_H */
