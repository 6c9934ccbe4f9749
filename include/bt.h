/*
 * bt.h - C ABI of the MI355X (gfx950) Block Transformer generation library.
 *
 * The library computes the batched autoregressive generation step of the Block
 * Transformer (arXiv 2406.02657): embedder lookup-and-concatenate (Sec. 2.2),
 * block decoder over a block-level KV cache, run once per L_B tokens
 * (Sec. 2.3), projection of the context embedding into prefix tokens and a
 * token decoder whose attention stays inside the current block (Sec. 2.4,
 * App. D.2 "Prefix"), LM head and greedy argmax; procedure per Sec. 2.1,
 * Fig. 1 and App. C (prefill runs the block decoder only; decoding emits one
 * token per sequence per step).  Layer type: Pythia / GPT-NeoX (Sec. 3.1).
 *
 * Conventions
 *   - "dev" pointers are HIP device pointers, "host" pointers ordinary memory.
 *   - The library allocates NO device memory: weights, token buffers, outputs
 *     and one workspace are caller-owned and must outlive the model.
 *   - All work is enqueued on the HIP stream given to bt_create and is
 *     asynchronous; outputs are valid once the caller synchronises that stream.
 *   - Every function returns BT_OK (0) or a negative bt_status.  Argument and
 *     state errors are detected on the host before anything is enqueued and
 *     leave the model unchanged.  No exceptions, no exit(); no state outside the
 *     models except the static workspace of bt_create_static and the text of the
 *     calling thread's last failed create call.
 *   - One model must not be used from two threads at once.
 *
 * Tensor layouts
 *   - Every linear map W is [out_features, in_features] row-major and is
 *     applied as y = x * W^T + b.  W_qkv rows: q (D), k (D), v (D); inside each
 *     part head h owns rows [h*d_head, (h+1)*d_head).  W_prefix is
 *     [P*D, D]; prefix token p is output slice [p*D, (p+1)*D).
 *   - dtype BT_F32: every tensor is float.  dtype BT_BF16: matrices and
 *     embedding tables (E_emb, E_tok, W_prefix, W_head, W_qkv, W_o, W_up,
 *     W_down) are bfloat16; biases and LayerNorm gamma/beta stay float.
 *     In bf16 mode GEMM operands and both KV caches are bf16; accumulation,
 *     residual stream, LayerNorm statistics, softmax and logits are float.
 */
#ifndef BT_H_
#define BT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BT_OK = 0,
  BT_ERR_ARG = -1,       /* null pointer, size out of range, unsupported shape */
  BT_ERR_STATE = -2,     /* decode before prefill, batch differs from prefill */
  BT_ERR_CAPACITY = -3,  /* block KV cache or workspace too small */
  BT_ERR_HIP = -4        /* HIP runtime error; text via bt_last_error */
} bt_status;

enum { BT_F32 = 0, BT_BF16 = 1 };
enum { BT_MIX_PREFIX = 0, BT_MIX_SUM = 1 };

/* Model and capacity description (plain data, filled by the caller).
 * Shape limits: d_model % n_heads == 0; d_head = d_model/n_heads in
 * {32, 64, 128}; d_model % block_len == 0 (d_emb = d_model/block_len, a
 * multiple of 8); rotary_dims even and <= d_head; prefix_len >= 1, or 0 with
 * block_len == 1 (then the context embedding itself is the token decoder's
 * single input row).  In bf16 mode d_model and d_ff must be multiples of 64. */
typedef struct {
  int32_t struct_size;      /* sizeof(bt_config) as the caller compiled it; the library rejects any
                               other value (BT_ERR_ARG), so a caller built against an older or newer
                               header fails at bt_create instead of being misread */
  int32_t vocab;
  int32_t block_len;        /* L_B */
  int32_t d_model;          /* D, both decoders */
  int32_t n_heads;
  int32_t d_ff;
  int32_t n_block_layers;
  int32_t n_token_layers;
  int32_t prefix_len;       /* P */
  int32_t dtype;            /* BT_F32 or BT_BF16 */
  int32_t max_batch;
  int32_t max_blocks;       /* block-KV capacity per sequence (prompt + generated blocks) */
  int32_t rotary_dims;      /* per head, even; 0 = no position rotation */
  int32_t parallel_residual;/* 1: x + Attn(LN1 x) + MLP(LN2 x); 0: sequential */
  int32_t prefill_rows;     /* prompt blocks processed per prefill chunk; 0 = default (16384) */
  int32_t act_split;        /* bf16 mode only: activations enter the MFMA GEMMs as hi + lo bf16 pairs
                               (about 16 mantissa bits): 0 never, 1 in decode steps, 2 also in prefill */
  int32_t use_graphs;       /* 1: decode steps are captured into HIP graphs (one per position in the
                               block) and replayed; 0: every launch is issued eagerly.  Capture needs
                               a stream other than the default (NULL) stream; with the default stream
                               the steps run eagerly and bt_stats.graph_fallback is set */
  int32_t pad_id;           /* token id that fills, from the left, the first block of a prompt whose
                               length is not a multiple of L_B (App. "Random length padding"; the
                               paper does not name the id); 0 <= pad_id < vocab */
  int32_t score_rows;       /* 0: no scoring support.  > 0: bt_score may be called; it runs the LM head
                               over this many rows at a time (workspace: score_rows * vocab floats,
                               plus local KV for every block of a prefill chunk) */
  int32_t eos_id;           /* -1: none.  Otherwise a sequence that has emitted this id emits it at
                               every later step as well (the paper generates a fixed number of
                               tokens and states no stopping rule; the batch is static, so a finished
                               sequence still occupies its rows) */
  int32_t keep_logits;      /* 1: every decode step stores its float logits [batch, vocab] for
                               bt_get_logits.  0: the LM head skips that store wherever greedy argmax
                               works from the per-tile candidates the head leaves (bf16 mode);
                               bt_get_logits then returns BT_ERR_STATE */
  int32_t token_mix;        /* how the context embedding enters the token decoder (App. D.2):
                               BT_MIX_PREFIX: projected to prefix_len prefix tokens (the paper's design);
                               BT_MIX_SUM: projected to L_B vectors of dimension D, vector k added to the
                               token decoder's input at local position k ("Summation").  The paper does
                               not say what stands under vector 0, the position that predicts the
                               block's first token: here nothing does (input 0 is vector 0 alone), and
                               position k >= 1 holds E_tok[token k-1 of the block] + vector k.
                               W_prefix is then [L_B*D, D]; prefix_len must be 1 (it only sizes nothing);
                               bt_score is not available */
  float   ln_eps;
} bt_config;

/* Device pointers of one transformer layer (dtype as described above). */
typedef struct {
  const void *ln1_g, *ln1_b;     /* [D] float */
  const void *W_qkv, *b_qkv;     /* [3D, D], [3D] */
  const void *W_o,   *b_o;       /* [D, D],  [D]  */
  const void *ln2_g, *ln2_b;     /* [D] float */
  const void *W_up,  *b_up;      /* [F, D],  [F]  */
  const void *W_down,*b_down;    /* [D, F],  [D]  */
} bt_layer_weights;

typedef struct {
  const void *E_emb;             /* [V, D/L_B]  embedder table (Sec. 2.2) */
  const void *E_tok;             /* [V, D]      token decoder table (Sec. 2.4); unused when L_B == 1 */
  const void *W_prefix;          /* [P*D, D]    context -> prefix tokens (App. D.2); NULL when P == 0.
                                    BT_MIX_SUM: [L_B*D, D], context -> the L_B summands */
  const void *b_prefix;          /* [P*D] float (BT_MIX_SUM: [L_B*D]) */
  const void *W_head;            /* [V, D]      classifier, no bias */
  const void *blk_lnf_g, *blk_lnf_b;   /* final LayerNorm of the block decoder, [D] float */
  const void *tok_lnf_g, *tok_lnf_b;   /* final LayerNorm of the token decoder, [D] float */
  const bt_layer_weights *block_layers;  /* host array [n_block_layers] of device pointers */
  const bt_layer_weights *token_layers;  /* host array [n_token_layers] */
} bt_weights;

/* Counters of the procedure (host side, updated as work is enqueued). */
typedef struct {
  int64_t block_passes;        /* block-decoder passes, counted per block (prefill: N_p) */
  int64_t token_passes;        /* token-decoder invocations (0 right after prefill) */
  int64_t token_rows;          /* rows pushed through the token decoder, per sequence */
  int64_t block_kv_rows_read;  /* cached block entries attended by decode steps, per sequence */
  int64_t block_kv_bytes_read; /* same, in bytes over batch, layers, K and V */
  int32_t n_blocks;            /* entries now in the block KV cache (N) */
  int32_t r;                   /* tokens already generated in the open block */
  int32_t batch;               /* batch of the last prefill, 0 before */
  int32_t local_kv_high_water; /* most local KV entries ever live in one block */
  /* profiling (bt_set_profile): summed HIP-event time of the block-decoder
   * decode attention launches and their count since the last reset */
  double  attn_block_ms;
  int64_t attn_block_launches;
  int64_t attn_block_bytes;    /* algorithmic K+V bytes those launches streamed */
  /* same for the grouped projection GEMM launches of the decode steps (QKV+MLP-up, O+MLP-down;
   * parallel-residual wiring, bf16 mode) */
  double  gemm_decode_ms;
  int64_t gemm_decode_launches;
  int64_t gemm_decode_bytes;   /* weight bytes those launches read (each weight once) */
  /* same for the GEMM launches that finish their own epilogue (more than 256 rows: prefill and
   * bt_score; parallel-residual wiring): the grouped layer GEMMs and the LM head of bt_score */
  double  gemm_tiled_ms;
  int64_t gemm_tiled_launches;
  int64_t gemm_tiled_flops;    /* 2 * rows * N * K summed over those launches (one activation plane) */
  /* HIP-graph state of the decode steps (cfg.use_graphs) */
  int64_t graph_launches;      /* decode steps that ran as a graph replay since bt_create */
  int32_t graph_captures;      /* step kinds captured and instantiated so far */
  int32_t graph_fallback;      /* 1: capture or instantiation failed (or the stream is the default
                                  stream) and every later step is launched eagerly; the reason is in
                                  bt_last_error */
} bt_stats;

typedef struct bt_model bt_model;

/* Bytes of device workspace bt_create needs for this config (block KV cache,
 * local KV cache, activations, split-K partials, logits, argmax candidates and,
 * in bf16 mode, a second copy of every GEMM weight matrix in the order the
 * decode GEMMs fetch it: about the size of the model again; with
 * score_rows > 0 also the scoring buffers, and activation rows for one
 * sequence's blocks times prefix_len + L_B - 1).  host out pointer. */
int bt_workspace_bytes(const bt_config *cfg, size_t *bytes);

/* Build a model.  cfg, w: host structs (copied).  workspace_dev: device memory
 * of at least bt_workspace_bytes, 256-byte aligned, owned by the caller.
 * hip_stream: a hipStream_t (NULL = the default stream).  *out receives the
 * handle.  In bf16 mode the call reads every GEMM weight matrix once (a small
 * kernel writes the re-ordered copy into the workspace), fills the rotary
 * table and synchronises the stream; weights changed afterwards are not seen
 * by the decode steps.
 * Errors: BT_ERR_ARG (bad config / null), BT_ERR_CAPACITY (workspace too
 * small), BT_ERR_HIP. */
int bt_create(const bt_config *cfg, const bt_weights *w, void *workspace_dev,
              size_t workspace_bytes, void *hip_stream, bt_model **out);

/* bt_create for callers that cannot allocate device memory (code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): the workspace is a static device array inside the library,
 * BT_STATIC_WORKSPACE_BYTES per GPU, held from library load to process end.
 * The call allocates no device memory and calls no HIP allocation routine
 * (the handle is a small host object); a model made by it never allocates
 * later either: cfg.use_graphs is taken as 0 (graph instantiation allocates)
 * and profiling events exist only after bt_set_profile(1).  The device is the
 * one current at the call.  The array is shared by every call on that GPU and
 * keeps the last model's contents; nothing in it is assumed to be zero (bt_create
 * rewrites the tables, bt_prefill resets all sequence state).  Two live models
 * on one GPU would race on it, so the call refuses while one exists:
 * BT_ERR_STATE until bt_destroy of the earlier one (which waits for its
 * stream).  Errors: BT_ERR_CAPACITY if bt_workspace_bytes(cfg) exceeds
 * BT_STATIC_WORKSPACE_BYTES; otherwise as bt_create; text via
 * bt_last_error(NULL). */
#define BT_STATIC_WORKSPACE_BYTES (32u << 20)
int bt_create_static(const bt_config *cfg, const bt_weights *w, void *hip_stream, bt_model **out);

/* Prefill (Fig. 1; Sec. 2.4; App. C): run the embedder and the block decoder
 * over all prompt blocks, fill the block KV cache with ceil(prompt_len/L_B)
 * entries per sequence and keep the context embedding for the first generated
 * block.  The token decoder is not run.  Resets all sequence state
 * (re-entrant).  A prompt_len that is not a multiple of L_B (App. "Random
 * length padding"; footnote of the zero-shot table, Sec. 3) counts as the
 * prompt preceded by (-prompt_len mod L_B) copies of cfg.pad_id: the pads are
 * embedded into the first block like any other token; the caller's buffer
 * holds the unpadded ids only.  prompt_len == 1 is the paper's setting
 * without an input sequence (L_B - 1 pads and one token).
 * tokens_dev: int32 [batch, prompt_len] row-major, device; ids are not
 * range-checked.  Errors: BT_ERR_ARG if batch < 1, batch > max_batch or
 * prompt_len < 1; BT_ERR_CAPACITY if ceil(prompt_len/L_B) > max_blocks. */
int bt_prefill(bt_model *m, const int32_t *tokens_dev, int32_t batch, int32_t prompt_len);

/* Prefill of prompts of different lengths in one batch (same passages as
 * bt_prefill).  tokens_dev: int32 [batch, max_len] row-major, device; sequence
 * b holds its lens_host[b] ids at the start of row b, the rest of the row is
 * not read.  lens_host: host array [batch], 1 <= lens_host[b] <= max_len, read
 * before the call returns (the call synchronises the stream once to upload
 * it).  Every sequence is left-padded with cfg.pad_id to whole blocks on its
 * own, exactly as bt_prefill would pad it alone, so all sequences end on a
 * block boundary and the decode steps run in lockstep; sequence b starts with
 * ceil(lens_host[b]/L_B) cached blocks.  Results per sequence equal those of a
 * batch of that sequence alone.  The per-sequence counters of bt_stats
 * (n_blocks, block_passes, block_kv_rows_read) then describe the longest
 * sequence; the byte counters sum over the batch.
 * Errors: as bt_prefill; BT_ERR_ARG if a length lies outside [1, max_len]. */
int bt_prefill_ragged(bt_model *m, const int32_t *tokens_dev, const int32_t *lens_host,
                      int32_t batch, int32_t max_len);

/* One decode step (Sec. 2.1): emits exactly one token per sequence.  At the
 * first step of a block the finished block is embedded and pushed through the
 * block decoder (attention over the whole block KV cache), its context
 * embedding is projected to the prefix and the token decoder runs over the
 * prefix rows; at the other steps the token decoder runs over one row per
 * sequence with attention over the current block's local KV only.  Then LM
 * head and greedy argmax (lowest index on ties).
 * next_ids_dev: int32 [batch], device, receives the tokens.
 * Errors: BT_ERR_STATE before prefill or if batch differs from the prefill's;
 * BT_ERR_CAPACITY if the step needs a block slot >= max_blocks. */
int bt_decode_step(bt_model *m, int32_t batch, int32_t *next_ids_dev);

/* Teacher-forced scoring (Sec. 2.1, Fig. 1: block decoder and token decoder over
 * all blocks of a sequence at once; the token decoder sees each block as an
 * independent sequence of prefix_len + L_B - 1 rows).  tokens_dev: int32
 * [batch, len] row-major, device; len > L_B.  A len that is not a multiple of
 * L_B counts as left-padded with cfg.pad_id, as in bt_prefill.
 * nll_dev: float [batch, len], device; entry t receives
 * -log p(x_t | x_<t), the log-softmax of the logits the generation step would
 * produce at that position given the same history; the tokens of the first
 * block (the first L_B - pads of them) have no context embedding and get 0.  Needs cfg.score_rows > 0 and prefix_len >= 1.
 * Overwrites the block KV cache: any generation in progress is lost (a new
 * bt_prefill is needed before bt_decode_step).  Errors: BT_ERR_ARG (null,
 * sizes), BT_ERR_STATE (score_rows == 0), BT_ERR_CAPACITY (ceil(len / L_B) >
 * max_blocks, or one sequence's rows exceed the workspace), BT_ERR_HIP. */
int bt_score(bt_model *m, const int32_t *tokens_dev, int32_t batch, int32_t len, float *nll_dev);

/* End-of-sequence flags (for callers that stop early; no passage of the paper:
 * it times a fixed number of generated tokens).  flags_dev: int32 [batch],
 * device; flags_dev[b] = 1 once sequence b has emitted cfg.eos_id at some
 * step since the last prefill, else 0 (always 0 when eos_id == -1).  Enqueued
 * on the model's stream like every other call.  Errors: BT_ERR_ARG (null),
 * BT_ERR_STATE (no prefill yet). */
int bt_get_finished(bt_model *m, int32_t *flags_dev);

/* Embedder alone (Sec. 2.2; App. D.1 "Lookup"): out_dev[m, j*d_emb + e] =
 * E_emb[tokens_dev[m*L_B + j], e] widened to float.  tokens_dev: int32
 * [n_rows, L_B], out_dev: float [n_rows, D], both device.  Does not touch the
 * sequence state.  Errors: BT_ERR_ARG on null pointers or n_rows < 0. */
int bt_embed(bt_model *m, const int32_t *tokens_dev, int32_t n_rows, float *out_dev);

/* Copy the float logits [batch, vocab] of the last decode step to logits_dev
 * (device), on the model's stream.  For parity checks.  Errors: BT_ERR_STATE if
 * no decode step has run since the last prefill, or cfg.keep_logits == 0. */
int bt_get_logits(bt_model *m, float *logits_dev);

/* Replace the token that the last decode step appended to each sequence's
 * history (teacher forcing for parity checks).  ids_dev: int32 [batch], device.
 * Must follow a bt_decode_step and precede the next one (else BT_ERR_STATE).
 * With cfg.eos_id >= 0 a forced eos_id marks the sequence finished, as an
 * emitted one does. */
int bt_force_last_ids(bt_model *m, const int32_t *ids_dev);

/* Copy the current context embedding [batch, D] (model dtype) out / in, on the
 * model's stream (locality checks inject a context).  Device pointers. */
int bt_get_context(bt_model *m, void *ctx_dev);
int bt_set_context(bt_model *m, const void *ctx_dev);

/* Profiling: when on, HIP events bracket every block-decoder decode attention
 * launch and every grouped projection GEMM launch of the decode steps, and the
 * steps are launched eagerly (no graph replay); bt_get_stats (which then
 * synchronises the stream) reports the sums.
 * bt_reset_profile clears the sums. */
int bt_set_profile(bt_model *m, int32_t on);
int bt_reset_profile(bt_model *m);

/* Calibration probes for the benchmark's "measured achievable" peaks (no model
 * needed; the caller times the launch with HIP events on hip_stream):
 *   bt_probe_read streams `bytes` bytes at src_dev (device; a multiple of
 *     BT_PROBE_READ_GRAIN) through BT_PROBE_WORKGROUPS workgroups with 16-byte
 *     loads and leaves one word per workgroup in out_dev: a plain read of HBM.
 *   bt_probe_mfma makes every wave of BT_PROBE_WORKGROUPS workgroups x 4 waves
 *     issue iters x 64 bf16 MFMAs (16 x 16 x 32) on 16 independent accumulators
 *     and nothing else: BT_PROBE_WORKGROUPS * 4 * iters * 64 * 16384 flops.
 *     random_operands != 0 gives every lane pseudo-random operand values (the
 *     clock the chip holds depends on the data); 0 gives constants.
 * out_dev: device, at least BT_PROBE_WORKGROUPS * 256 floats, overwritten.
 * Errors: BT_ERR_ARG, BT_ERR_HIP. */
#define BT_PROBE_WORKGROUPS 2048
#define BT_PROBE_READ_GRAIN ((size_t)BT_PROBE_WORKGROUPS * 256 * 16)
int bt_probe_read(const void *src_dev, size_t bytes, void *hip_stream, float *out_dev);
int bt_probe_mfma(int32_t iters, int32_t random_operands, void *hip_stream, float *out_dev);

int bt_get_stats(bt_model *m, bt_stats *out);

/* Text of the last error on this model (host string owned by the model).  With
 * m == NULL: why the calling thread's last bt_create / bt_create_static failed. */
const char *bt_last_error(const bt_model *m);

void bt_destroy(bt_model *m);

#ifdef __cplusplus
}
#endif
#endif /* BT_H_ */
