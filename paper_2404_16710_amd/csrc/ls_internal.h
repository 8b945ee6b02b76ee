// Shared between the host side of the C ABI (ls_api.cpp) and the device code (ls_kernels.hip).
#ifndef LS_INTERNAL_H_
#define LS_INTERNAL_H_

#include <stdint.h>
#include <stddef.h>

#define LS_THREADS 256          // workgroup size of the persistent kernel (4 wavefronts)
#define LS_WAVES (LS_THREADS / 64)
#define LS_SLOTS 4              // 256-byte weight blocks per wave kept in flight (per tile: LS_SLOTS / tiles)
#define LS_ROWS 16              // rows per pass (MFMA N dimension)
#define LS_ATTN_TILE 64         // KV positions per attention work item
#define LS_ACT_BYTES (128 * 1024) // LDS bytes for staged matmul inputs
#define LS_MISC_BYTES 6656       // LDS bytes for state, statistics and small scratch
#define LS_RED_BYTES 8192        // LDS bytes for the cross-wave reduction of accumulator tiles
#define LS_SMEM_BYTES (LS_ACT_BYTES + LS_RED_BYTES + LS_MISC_BYTES)

// Size of the library's own workspace array (ls_generate_static): enough for tiny models only.
#define LS_STATIC_SCRATCH_BYTES (8u << 20)

struct LsLayerW {
  const void *wq, *wk, *wv, *wo, *wg, *wu, *wd, *attn_norm, *ffn_norm;
};

// Decoding state.  One copy lives in device memory (read by the host through ls_get_state /
// ls_peek_round); every workgroup keeps an identical working copy in LDS while a program runs.
struct LsState {
  int32_t pos;         // KV positions that are final: prompt + emitted - 1
  int32_t last;        // last emitted token; not yet in the cache
  int32_t n_gen;       // tokens emitted so far
  int32_t done;        // generation finished (max_new reached or eos emitted)
  int32_t error;       // device-side error: 1 bounded wait expired, 2 capacity
  int32_t n_acc;       // drafts accepted in the last round
  int32_t draft_valid; // exit-state rows 0..draft_d hold the drafts of (draft_E, draft_d)
  int32_t draft_E, draft_d;
  int32_t n_emit;      // tokens the last round emitted (before the max_new cut)
  int64_t rounds, drafted, accepted;
  int64_t low_exits;   // drafts that left at the lower of two exit layers (per-token exit layer)
  int32_t D[LS_ROWS];
  int32_t V[LS_ROWS];
  float dmargin[LS_ROWS];
  float vmargin[LS_ROWS];
};

enum LsProgramKind {
  LS_PROG_PREFILL = 0,   // tokens[0..n) through layers 0..layers_used, head on the last row
  LS_PROG_SCORE = 1,     // same, head on every row, argmax/margin written per row
  LS_PROG_DRAFT = 2,
  LS_PROG_VERIFY = 3,
  LS_PROG_GENERATE = 4,  // rounds of draft+verify (d > 0) or single-token passes (d == 0)
  LS_PROG_PF_FINISH = 5  // GEMM prefill: head on residual row 0, then the state of a finished prefill
};

struct LsKParams {
  // model
  int32_t L, dm, nq, nkv, hd, ffn, vocab, qd, kvd, G, max_seq;
  float eps, attn_scale;
  const LsLayerW *layers;
  const void *embed, *final_norm, *lm_head;
  const float *rope_cos, *rope_sin; // [max_seq][hd/2]
  // workspace
  void *kcache, *vcache;            // [L][nkv][max_seq][hd]
  float *xbuf;                      // [16][dm]  residual rows = exit-state rows
  float *ssq;                       // [16][ssq_nt] sum of squares of xbuf rows, one slot per workgroup
  void *qbuf, *obuf, *actbuf;       // [16][qd], [16][qd], [16][ffn]
  float *attn_part;                 // [nkv][max_tiles][64][hd+2]
  uint32_t *attn_cnt;               // [nkv]
  int32_t max_tiles;
  int32_t attn_ctiles;              // 64-position tiles per attention work item (from the cache capacity)
  int32_t kv_through_caches;        // settled K/V tiles are read with cacheable loads: set when the whole KV cache
                                    // is small enough to stay in the memory-side cache between passes
  float *cand;                      // [grid][16][4]
  uint32_t *bar;                    // grid barrier counters (4096 bytes)
  LsState *state;
  float *capture;                   // [L][max_seq][dm] or null
  // ssq_nt: sums of squares per residual row (the number of workgroups); x_tiles: most weight tiles
  // a workgroup gets in the O / down projections (two of them share the staged input)
  int32_t ssq_nt, x_tiles;
  // program
  int32_t kind, E, d, max_new, eos, n_tokens, layers_used;
  int32_t probe;      // LS_PROG_SCORE: argmax of the head after every layer, outputs [layer][row]
  int32_t no_reuse;   // rounds verify with all L layers instead of continuing from the exit states (ablation)
  int32_t E_low;      // > 0: per-token exit layer, a draft leaves at E_low when its margin is at least tau, else at E
  float tau;
  int32_t *out_exits; // [rounds][d] exit layer of every draft, or null
  const int32_t *tokens;
  int32_t *out_tokens;
  float *out_margin;
  int32_t spin_limit;
  // optional timeline of one workgroup: (100 MHz wall clock << 8) | tag, appended per event
  unsigned long long *prof;
  int32_t prof_cap, prof_wg;
};

// Parameters of the GEMM prefill (host side launches; see ls_prefill.hip).
struct LsPfParams {
  int32_t is_bf16, dm, qd, kvd, ffn, vocab, hd, nkv, max_seq, layers_used;
  int32_t ssq_nt;              // sums of squares per residual row (LsKParams::ssq_nt)
  float eps;
  const int32_t *tokens;
  const void *embed;
  const float *rope_cos, *rope_sin;
  void *kcache, *vcache;
  float *x_pf;                 // [pf_rows][dm] residual rows of the chunk
  void *a_pf, *q_pf, *o_pf, *act_pf;  // [pf_rows][dm], [..][qd], [..][qd], [..][ffn] in the model dtype
  float *xbuf, *ssq;           // decode residual row 0 and its statistics (target of the finish step)
  float *capture;
  int32_t tile_rows;           // rows of a prompt GEMM's output tile: 0 = by the number of tiles, else 32, 64 or 128
};

#endif
