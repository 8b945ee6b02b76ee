/*
 * ls.h - C ABI of the MI355X (gfx950) library for greedy self-speculative decoding with
 * early-exit drafts on a Llama-style decoder, batch 1, one GPU.
 *
 * Method (paper sections, restated in our words):
 *   - Section 4.1: the decoder is x_{l+1} = x_l + f_l(x_l) for l = 0..L-1; the LM head g is the
 *     final normalisation followed by the final linear layer (Section 2.1) and is shared by
 *     every exit.
 *   - Section 4.2: an early exit at E runs layers 0..E-1 and predicts with g(x_E).
 *   - Section 4.3.1 (self-drafting): d tokens are drafted autoregressively with the early exit.
 *   - Section 4.3.2 (self-verification): layers E..L-1 predict, in one pass, the token after
 *     each of the 1+d rows (the round's input token and the d drafts); drafts are kept up to
 *     the first disagreement and the verified token at that point is appended.
 *   - Section 4.3.3 (cache reuse): one KV cache for both stages, plus the exit-layer states of
 *     the drafted positions so that verification starts at layer E.
 *   - Appendix A.4: after a round the cache keeps (prompt + emitted - 1) positions.
 *
 * Conventions
 *   - Pointers marked DEVICE point to GPU memory the CALLER owns (weights, workspace, token
 *     buffers).  The library never allocates or frees device memory.  Pointers marked HOST are
 *     ordinary host memory.  `stream` is a hipStream_t passed as void* (NULL = default stream).
 *   - Matrices are row-major [out_features, in_features]; dtype is LS_F32 or LS_BF16 for all
 *     weights, the KV cache and the matmul inputs; accumulation, the residual stream, softmax
 *     and logits are fp32.
 *   - Every function returns LS_OK (0) or a negative LS_E_* code; none aborts or throws.
 *     Arguments are validated before anything is enqueued, so LS_E_ARG / LS_E_RANGE /
 *     LS_E_CAPACITY / LS_E_STATE never leave work on the stream.
 *   - ls_prefill / ls_draft / ls_verify only ENQUEUE on `stream`; their results live in device
 *     state.  ls_generate, ls_score, ls_get_state and ls_peek_round synchronise the stream.
 *   - One context is one sequence: calls on one context must not overlap in time.
 */
#ifndef LS_H_
#define LS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ls_ctx ls_ctx; /* opaque host object */

enum { LS_F32 = 0, LS_BF16 = 1 };

enum {
  LS_OK = 0,
  LS_E_ARG = -1,      /* null pointer, unsupported shape or dtype                           */
  LS_E_RANGE = -2,    /* exit_layer outside [1, L], d outside [0, max_draft], bad counts    */
  LS_E_CAPACITY = -3, /* workspace too small, or the sequence would not fit in max_seq      */
  LS_E_STATE = -4,    /* call order: draft before prefill, verify without a matching draft  */
  LS_E_HIP = -5,      /* a HIP runtime call failed                                          */
  LS_E_DEVICE = -6    /* the device reported an error (bounded wait expired, capacity)      */
};

#define LS_MAX_ROWS 16 /* rows per pass: 1 + max_draft <= 16 */

typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, vocab;
  float rope_base, rms_eps;
  int32_t dtype;     /* LS_F32 or LS_BF16                                                   */
  int32_t max_seq;   /* KV capacity in positions, at most 32768                             */
  int32_t max_draft; /* 1..15                                                               */
} ls_config;
/* Supported shapes: head_dim 64 or 128; n_q_heads a multiple of n_kv_heads with ratio <= 4;
 * d_model, ffn_dim, n_q_heads*head_dim multiples of 16; vocab a multiple of 16. */

typedef struct { /* all DEVICE pointers; the per-layer arrays are HOST arrays of DEVICE pointers */
  const void *embed;                                  /* [vocab, d_model]                   */
  const void *const *wq, *const *wk, *const *wv;      /* [n_q*hd, dm], [n_kv*hd, dm] x2      */
  const void *const *wo;                              /* [dm, n_q*hd]                        */
  const void *const *w_gate, *const *w_up;            /* [ffn, dm]                           */
  const void *const *w_down;                          /* [dm, ffn]                           */
  const void *const *attn_norm, *const *ffn_norm;     /* [dm] RMSNorm gains                  */
  const void *final_norm;                             /* [dm]                                */
  const void *lm_head;                                /* [vocab, dm] (not tied to embed)     */
} ls_weights;

typedef struct {
  int64_t rounds;    /* draft+verify rounds run (0 for full-model greedy)                    */
  int64_t drafted;   /* d per round                                                          */
  int64_t accepted;  /* drafts kept by verification; acceptance rate = accepted / drafted    */
  int64_t generated; /* tokens written to the output                                         */
  float ms_prefill;  /* device time of the prefill, from events on `stream`                  */
  float ms_decode;   /* device time of everything after the prefill                          */
} ls_stats;

/* Bytes of DEVICE workspace ls_load_weights needs for this configuration (KV cache, exit-state
 * rows, per-stage scratch, rotary table, device state).  0 if the configuration is invalid. */
size_t ls_workspace_bytes(const ls_config *cfg);

/* Creates a context.  `weights` pointers are kept (not copied) and must outlive the context;
 * `dev_workspace` (DEVICE, 256-byte aligned, >= ls_workspace_bytes) is owned by the caller and
 * used exclusively by this context.  Uploads the rotary table and the layer pointer table into
 * the workspace (synchronously) and zeroes the device state.  *out is the new context. */
int ls_load_weights(const ls_config *cfg, const ls_weights *weights, void *dev_workspace,
                    size_t workspace_bytes, ls_ctx **out);

/* Prefill: all L layers over the n_prompt prompt ids (DEVICE int32[n_prompt]); fills the KV cache
 * at positions [0, n_prompt) and takes the first generated token t_0 = argmax g(x_L[n_prompt-1]).
 * Resets the decoding state to {pos = n_prompt, last = t_0, n_gen = 1}.  Enqueue only.
 * The prompt buffer must stay valid until the stream has run the call. */
int ls_prefill(ls_ctx *ctx, const int32_t *dev_prompt, int32_t n_prompt, void *stream);

/* Self-drafting (Section 4.3.1): d early-exit steps through layers 0..exit_layer-1, each followed
 * by the shared head and an argmax, giving D_0..D_{d-1}; then the early layers once more for
 * D_{d-1} (no head), so that the exit-state rows 0..d are complete.  Appends K,V of layers
 * < exit_layer at positions pos..pos+d.  Enqueue only.  d >= 1. */
int ls_draft(ls_ctx *ctx, int32_t exit_layer, int32_t d, void *stream);

/* Self-verification (Section 4.3.2) + acceptance + cache crop (Appendix A.4): layers
 * exit_layer..L-1 over the 1+d exit-state rows in one pass, head + argmax per row giving
 * V_0..V_d; n = number of leading drafts with D_i == V_i; the round emits D_0..D_{n-1}, V_n;
 * pos += n+1, last = V_n.  Must follow ls_draft with the same (exit_layer, d).  Enqueue only. */
int ls_verify(ls_ctx *ctx, int32_t exit_layer, int32_t d, void *stream);

/* Whole job: prefill, then rounds of draft+verify until max_new tokens exist (the first comes
 * from the prefill), all enqueued without host round-trips; d = 0 runs full-model greedy
 * decoding instead (the autoregressive baseline).  Stops early after emitting eos_id (pass -1
 * for none).  dev_out_tokens: DEVICE int32[max_new], unused tail filled with -1.
 * host_stats (HOST, may be NULL) receives the counters.  Synchronises `stream`. */
int ls_generate(ls_ctx *ctx, const int32_t *dev_prompt, int32_t n_prompt, int32_t max_new,
                int32_t exit_layer, int32_t d, int32_t eos_id, int32_t *dev_out_tokens,
                ls_stats *host_stats, void *stream);

/* Ablation of the shared cache and exit states (Section 4.3.3; the cache-reuse table of the
 * appendix): same arguments, output tokens and statistics as ls_generate with d >= 1, but every
 * round verifies with ALL layers over its 1+d tokens instead of continuing from the exit-layer
 * states and early-layer cache the draft stage left (and skips the early-layer pass of the last
 * draft, which only exists to feed that continuation).  The difference in time is what the reuse saves. */
int ls_generate_no_reuse(ls_ctx *ctx, const int32_t *dev_prompt, int32_t n_prompt, int32_t max_new,
                         int32_t exit_layer, int32_t draft_len, int32_t eos_token,
                         int32_t *dev_out_tokens, ls_stats *host_stats, void *stream);

/* Self-speculative decoding with a per-token exit layer, the extension the paper's closing section
 * names as future work (an exit layer chosen per token by a condition evaluated while decoding);
 * the paper gives no algorithm, the reading implemented is: a draft leaves at layer exit_low when the margin between
 * the two largest logits of g(x_{exit_low}) is at least tau, otherwise it continues to exit_high
 * (1 <= exit_low < exit_high <= L); rows that left early pass through layers exit_low..exit_high-1
 * later, several rows per pass, so that verification (from exit_high, Section 4.3.2) and the
 * output tokens are exactly those of ls_generate(exit_layer = exit_high).  tau = +inf never leaves
 * early; tau <= 0 always does.  dev_exit_layers (DEVICE int32[max_new * d], or NULL) receives the
 * exit layer of every draft, round by round; *host_low_exits (HOST, or NULL) the number of drafts
 * that left at exit_low.  Otherwise as ls_generate with d >= 1. */
int ls_generate_dynamic(ls_ctx *ctx, const int32_t *dev_prompt, int32_t n_prompt, int32_t max_new,
                        int32_t exit_low, int32_t exit_high, int32_t draft_len, float tau,
                        int32_t eos_token, int32_t *dev_out_tokens, int32_t *dev_exit_layers,
                        ls_stats *host_stats, int64_t *host_low_exits, void *stream);

/* Early exit on its own (Section 4.2): like ls_generate with d = 0, but every pass, the prefill
 * included, runs layers 0..exit_layer-1 only and predicts with g(x_E). */
int ls_generate_early_exit(ls_ctx *ctx, const int32_t *dev_prompt, int32_t n_prompt,
                           int32_t max_new, int32_t exit_layer, int32_t *dev_out_tokens,
                           ls_stats *host_stats, void *stream);

/* Inspection: teacher-forced scoring.  Runs layers 0..n_layers_used-1 (1..L) over n tokens
 * (DEVICE int32[n]) as one causal sequence from position 0 and writes, for every row, the argmax
 * of g(x) (DEVICE int32[n]) and, if dev_margin is not NULL, top-1 minus top-2 of its logits
 * (DEVICE float[n]).  Overwrites the KV cache and invalidates the decoding state.  Synchronises. */
int ls_score(ls_ctx *ctx, const int32_t *dev_tokens, int32_t n, int32_t n_layers_used,
             int32_t *dev_argmax, float *dev_margin, void *stream);

/* The unembedding probe of Section 3 (which layer first predicts the final token): like ls_score
 * over all layers, but the shared head g is applied to the output of EVERY layer.  dev_argmax is
 * DEVICE int32[n_layers][n], dev_margin DEVICE float[n_layers][n] or NULL; row l holds argmax g(x_{l+1}).
 * Overwrites the KV cache and invalidates the decoding state.  Synchronises. */
int ls_probe_layers(ls_ctx *ctx, const int32_t *dev_tokens, int32_t n, int32_t *dev_argmax,
                    float *dev_margin, void *stream);

/* Inspection: synchronises `stream` and returns the decoding state (HOST out-pointers, any may
 * be NULL).  Returns LS_E_DEVICE if the device flagged an error. */
int ls_get_state(ls_ctx *ctx, int32_t *pos, int32_t *last, int32_t *n_gen, void *stream);

/* Inspection: synchronises and copies out the last round: drafts (HOST int32[d]), verified
 * tokens (HOST int32[d+1]), their logit margins (HOST float[d], float[d+1]; may be NULL) and the
 * number of accepted drafts. */
int ls_peek_round(ls_ctx *ctx, int32_t *host_draft, int32_t *host_verify, float *host_draft_margin,
                  float *host_verify_margin, int32_t *n_accept, void *stream);

/* Inspection: from now on every pass also stores x_{l+1} of each row it computes at
 * dev_hidden[l][position][:] (DEVICE float [n_layers][max_seq][d_model]); NULL switches it off. */
int ls_debug_capture(ls_ctx *ctx, float *dev_hidden);

/* Inspection: from now on every launch appends the timeline of one workgroup to dev_events (DEVICE
 * uint64[capacity], each entry (100 MHz device clock << 8) | stage tag, restarting at entry 0 per
 * launch); NULL switches it off.  Used to see where a pass spends its time. */
int ls_debug_timeline(ls_ctx *ctx, unsigned long long *dev_events, int32_t capacity, int32_t workgroup);

/* Measurement aid: copies `bytes` (a multiple of 16; both pointers DEVICE, 16-byte aligned) with
 * a plain copy kernel (ls_copy_kernel).  Profilers use it as the known-size reference that hardware
 * byte counters are scaled by.  Enqueue only. */
int ls_debug_copy(void *dev_dst, const void *dev_src, size_t bytes, void *stream);

/* Measurement aid: reads `bytes` of DEVICE memory once and writes nothing but 16 bytes per thread to
 * `dev_sink` (DEVICE, at least workgroups * 4096 bytes; both pointers 16-byte aligned), in the launch
 * shape of the decode kernels: `workgroups` workgroups of 256 threads (1..4096; the decode kernels run
 * 256), each walking a contiguous share with 16-byte loads, 64 KB per workgroup in flight.  `bytes` must
 * be a multiple of workgroups * 65536.  Its rate is the practical ceiling of a stage's weight stream
 * (ls_read_kernel in a profiler's kernel trace).  Enqueue only; LS_E_ARG on a bad argument. */
int ls_debug_read(const void *dev_src, size_t bytes, void *dev_sink, int32_t workgroups, void *stream);

/* Debug aid: how many polls a workgroup spends in one wait for the others before it gives up
 * (0 restores the default of about four million).  When a wait expires every workgroup leaves, the
 * call that launched the kernel returns LS_E_DEVICE, and the next ls_prefill / ls_generate* / ls_score
 * starts from rebuilt counters.  A limit of 1 makes that path testable without a hung kernel. */
int ls_debug_spin_limit(ls_ctx *ctx, int32_t polls);

/* Debug aid: how later calls read K/V tiles that no pass of the current round writes.  0 (default): with
 * cacheable loads when the whole KV cache of the configuration is at most 192 MB (it then survives in the
 * memory-side cache from pass to pass), with coherent loads otherwise; 1: always cacheable; 2: always
 * coherent.  The bytes read and the arithmetic are the same either way; the setting selects one of two
 * instantiations of the attention stage, and tests use it to run both on one model.  LS_E_RANGE otherwise. */
int ls_debug_kv_policy(ls_ctx *ctx, int32_t policy);

/* Launch shape: workgroups per compute unit used by later calls, from 1 to what the kernels' LDS and
 * register footprint lets a compute unit hold (the occupancy the runtime reports at load time; 1 with
 * the present 142 KB of LDS per workgroup); 0 restores the default, the maximum.  Returns the number
 * of workgroups a launch will use, or LS_E_RANGE for a count the device cannot keep resident. */
int ls_set_launch(ls_ctx *ctx, int32_t workgroups_per_cu);

/* Shape of the prompt pass used by later calls.  Prompts of 32 or more ids run as GEMMs over all
 * rows of a chunk, with output tiles of 128, 64 or 32 rows chosen from the number of tiles the
 * launch would have (rows = 0, the default); 32, 64 or 128 force that tile height, 160 forces 64-row
 * tiles that are 160 instead of 128 columns wide in the products into the residual rows (where 160
 * divides d_model; the default picks them when they fill the chip in fewer rounds), 16 sends every
 * prompt through the 16-row passes of the decode kernel.  All choices compute the same operation
 * and differ in the order of the floating-point sums only.  Host state only: no GPU work.
 * Returns LS_OK, LS_E_ARG for a null context or LS_E_RANGE for any other value. */
int ls_set_prompt_tiles(ls_ctx *ctx, int32_t rows);

/* For callers that cannot allocate device memory (code under HIP graph capture set-up, tight serving
 * loops, harnesses that forbid hipMalloc): ls_generate without a caller workspace and without a
 * context.  The KV cache and every per-stage buffer live in a fixed array inside the library
 * (ls_static_workspace_limit() bytes, 8 MiB, held by every GPU the library runs on until the process
 * ends), so the call allocates no device memory at all; it serves models whose
 * ls_workspace_bytes(cfg) fits that array (tiny models) and returns LS_E_CAPACITY, before touching
 * the device, for any other.  cfg / weights as for ls_load_weights (DEVICE weight pointers, kept only
 * for the duration of the call), the remaining arguments and the results as for ls_generate.
 * The array keeps the previous call's contents; every call rebuilds the tables, counters and state
 * it needs, so successive calls with different configurations are independent.  All calls on one
 * GPU share the one array: calls that overlap in time on the same GPU race and give undefined
 * results (serialise them; calls on different GPUs do not interact).  Synchronises `stream`. */
int ls_generate_static(const ls_config *cfg, const ls_weights *weights, const int32_t *dev_prompt,
                       int32_t n_prompt, int32_t max_new, int32_t exit_layer, int32_t d, int32_t eos_id,
                       int32_t *dev_out_tokens, ls_stats *host_stats, void *stream);
size_t ls_static_workspace_limit(void);

const char *ls_strerror(int code);

/* Frees the host object only; the workspace and the weights stay with the caller. */
void ls_destroy(ls_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* LS_H_ */
