// Host-side launchers of the gfx950 kernels.  Every launcher enqueues on the
// given stream and returns hipGetLastError().  `dtype` is BT_F32 or BT_BF16 and
// selects the storage type of matrices, GEMM operands and KV caches.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace bt {

// ---------------------------------------------------------------- elementwise
// Embedder (Sec. 2.2): row m = b * blocks_per_seq + i of x is the concatenation of the table rows
// of block i of sequence b, float out.  tokens [n_seqs, row_stride]; sequence b holds seq_lens[b]
// ids (seq_lens null: seq_len for all) at the start of its row and counts as left-padded with
// pad_id to the next multiple of L_B (App. "Random length padding").  Blocks past a sequence's
// own end (shorter sequences of a batch) are filled with pad_id; their rows are never used.
hipError_t launch_embed_concat(int dtype, const void* E_emb, const int32_t* tokens, float* x,
                               int n_seqs, int blocks_per_seq, int block_len, int d_emb,
                               int row_stride, int seq_len, const int* seq_lens, int pad_id, hipStream_t s);

// Token-decoder input row: x[b, :] = E_tok[cur[b*L_B + r_prev], :], float out.
hipError_t launch_token_embed(int dtype, const void* E_tok, const int32_t* cur, float* x,
                              int batch, int block_len, int r_prev, int d_model, hipStream_t s);

// Residual update + LayerNorm(s) of one row per workgroup.
//   in row  = i * in_mul + in_off   (for x and the partial sums)
//   x_new   = x + (biasA + sum_s partA[s]) + (biasB + sum_s partB[s])
//   u1[i]   = LN(x_new; g1, b1)  (storage dtype, or float when u1_f32)
//   u2[i]   = LN(x_new; g2, b2)  (optional)
struct ResidLnArgs {
  float* x;              // [*, D] residual stream (updated in place when write_x)
  const float* partA;    // [splitsA][part_rows][D] or null
  const float* biasA;
  int splitsA;
  const float* partB;
  const float* biasB;
  int splitsB;
  size_t part_stride;    // elements between consecutive splits
  const float *g1, *b1;
  void* u1;
  int u1_f32;
  const float *g2, *b2;  // null: no second output
  void* u2;
  int n_rows, D, in_mul, in_off, write_x;
  float eps;
  size_t lo_off;         // != 0: u1 / u2 also get the bf16 remainder plane at +lo_off elements
  // Optional: the rows do not come from x but from an embedding table (storage dtype, [*, D]):
  // row i = emb_table[emb_ids[i * emb_stride + emb_off]]; with write_x the residual stream gets them.
  const void* emb_table;
  const int32_t* emb_ids;
  int emb_stride, emb_off;
  // Optional: row i adds 1 to counter_inc[i] (the device-side count of cached blocks of sequence i).
  int* counter_inc;
  // Optional (summation token decoder, first launch of a stack): row i also gets the float vector
  // add[i * add_stride ...]; without emb_table the row is that vector alone (x is not read).
  const float* add;
  int add_stride;
};
// in_off_dev (optional, device memory): row i takes in_off_dev[i] - 1 in place of a.in_off.  It is
// a launch argument of its own, used by a separate instantiation: the size and field offsets of
// ResidLnArgs measurably change the cost of the decode-step launches.
hipError_t launch_resid_ln(int dtype, const ResidLnArgs& a, hipStream_t s, const int* in_off_dev = nullptr);

// Greedy argmax over logits [batch, vocab] (lowest index on ties); writes
// next_ids[b] (if non-null) and cur[b*L_B + r].  eos_id >= 0: once sequence b has emitted eos_id
// (finished[b] is then set, device memory), every later id of b is eos_id.
hipError_t launch_argmax(const float* logits, int batch, int vocab, int32_t* next_ids,
                         int32_t* cur, int block_len, int r, int eos_id, int32_t* finished, hipStream_t s);
// The same from per-tile candidates cand[b * n_tiles + tile] = (value, column as int bits); a column outside
// [0, vocab) counts as "no candidate" (id 0).
hipError_t launch_argmax_candidates(const float2* cand, int n_tiles, int batch, int vocab, int32_t* next_ids,
                                    int32_t* cur, int block_len, int r, int eos_id, int32_t* finished, hipStream_t s);

// cur[b*L_B + r] = ids[b]; with eos_id >= 0 also finished[b] = 1 where ids[b] == eos_id
hipError_t launch_scatter_ids(const int32_t* ids, int32_t* cur, int batch, int block_len, int r, int eos_id,
                              int32_t* finished, hipStream_t s);
// dst = src, `bytes` a multiple of 16, both 16-byte aligned
hipError_t launch_copy16(void* dst, const void* src, size_t bytes, hipStream_t s);
// out[b] = cur[b*L_B + r]
hipError_t launch_gather_ids(const int32_t* cur, int32_t* out, int batch, int block_len, int r, hipStream_t s);
// p[i] = value for i < n: the device-side counts of cached blocks, one per sequence
hipError_t launch_state_set(int* p, int value, int n, hipStream_t s);
// n_blocks[i] = ceil(lens[i] / block_len) for i < n
hipError_t launch_seq_blocks(const int* lens, int* n_blocks, int block_len, int n, hipStream_t s);

// Teacher-forced scoring (Sec. 2.1: every block of a sequence at once).  A chunk holds n_seqs
// sequences of seq_len tokens = n_blocks blocks once the first block is completed from the left with
// n_blocks * L_B - seq_len pads (token indices below count the pads); local sequence s = bl * (n_blocks - 1) + j scores block j + 1 of
// sequence bl from the context embedding of block j and has Lq = P + L_B - 1 rows.
// assemble: x[s * Lq + p] = pref[(bl * n_blocks + j), p * D ...] for p < P (prefix rows, float), then
// E_tok[tokens[bl * seq_len + (j + 1) * L_B + k]] for k < L_B - 1.  tokens: the chunk's first row.
hipError_t launch_score_assemble(int dtype, const float* pref, const void* E_tok, const int32_t* tokens, float* x,
                                 int n_seqs, int n_blocks, int seq_len, int D, int P, int block_len, hipStream_t s);
// logits [n_rows, vocab] of the chunk's rows row0 .. row0 + n_rows - 1 (row = s * Lq + pos).  Rows with
// pos >= P - 1 predict token k = pos - (P - 1) of their block: nll[bl * seq_len + (j + 1) * L_B + k] =
// log sum exp(logits) - logits[that token].  tokens, nll: the chunk's first row.
hipError_t launch_score_rows(const float* logits, int n_rows, int vocab, int row0, const int32_t* tokens, float* nll,
                             int P, int block_len, int n_blocks, int seq_len, hipStream_t s);

// The same without the logits: targets[row] = the token row `row` of the chunk predicts (-1: none), for a
// GEMM with the EPI_LSE epilogue; and the combination of what that GEMM leaves for rows row0 .. row0 +
// n_rows - 1: stats [n_rows][groups] (max, sum of exponentials), target_logit [n_rows].
hipError_t launch_score_targets(const int32_t* tokens, int32_t* targets, int n_rows, int P, int block_len,
                                int n_blocks, int seq_len, hipStream_t s);
hipError_t launch_score_combine(const float2* stats, int groups, const float* target_logit, int n_rows, int row0,
                                float* nll, int P, int block_len, int n_blocks, int seq_len, hipStream_t s);

// --------------------------------------------------------------- calibration probes
// A plain streaming read of `bytes` (a multiple of grid * 256 * 16) and a loop of nothing but MFMAs; one
// float per thread / workgroup lands in out so that nothing is optimised away.
hipError_t launch_probe_read(const void* src, size_t bytes, int workgroups, float* out, hipStream_t s);
hipError_t launch_probe_mfma(int iters, int random_operands, int workgroups, float* out, hipStream_t s);

// ----------------------------------------------------------------------- GEMM
enum { EPI_F32 = 0,        // out float [M, ldo]: acc + bias
       EPI_GELU = 1,       // out storage dtype: gelu(acc + bias)
       EPI_PARTIAL = 2,    // out float [splits][M][N]: raw partial sums (no bias); the consumer
                           // sums the splits in order and applies bias / activation
       EPI_QKV = 4,        // tiled bf16 kernels only, N = 3 D (q | k | v): the block decoder's prefill.  acc + bias,
                           // then per column region: q rotated (rotary) and stored float into out [M, ldo];
                           // k rotated, v as is, both stored in the storage dtype straight into the block KV
                           // cache (see QkvEpilogue); the k and v columns of `out` are not written
       EPI_LSE = 3 };      // tiled bf16 kernels only: the values acc + bias are not stored; out is
                           // float2 [M][ceil(N/64)]: per row and group of 64 columns (max, sum of
                           // exp(value - max)), and the value at column lse_targets[row] goes to
                           // lse_target_out[row] (rows whose target is negative write nothing)

// out[M, N] = A[M, K] * W[N, K]^T (+ bias).  A, W in the storage dtype, row-major,
// lda / K contiguous.
// A_lo (optional, bf16 mode): remainder plane of A, so that the product uses A + A_lo.
// out_lo_off (EPI_GELU, bf16 mode): != 0 stores the output as hi / remainder planes.
// W_frag (bf16 mode, required when M <= 256): the same weights in MFMA fragment order
// (see gemm_pack_weights); the decode kernel reads only this copy.
// EPI_QKV: row m of the GEMM is block position pos0 + m % n_new of sequence m / n_new.  Cache layout per
// layer: K [B][H][n_cap][d_head], V same; rope[pos * (rot/2) + t] = (cos, sin).  rot/2 must be 0, 8 or 16
// (gemm_qkv_epilogue_ok): the rotation partner of a column then sits in the same wave's accumulators.
struct QkvEpilogue {
  const float2* rope;
  void *Kc, *Vc;
  int n_new, pos0, n_heads, d_head, rot, n_cap;
};
bool gemm_qkv_epilogue_ok(int d_model, int d_head, int rot);

struct GemmProblem {
  const void* A;
  const void* W;
  const float* bias;
  void* out;
  int M, N, K, lda, ldo, epi;
  const void* A_lo;
  size_t out_lo_off;
  const void* W_frag;
  // EPI_F32, one K-split: when non-null, every workgroup (decode kernel, M <= 192) or wavefront (tiled
  // kernels: one per 64 columns) also writes, per row, the largest value of its columns and that column
  // (lowest on ties) to row_max[row * tiles + tile]; gemm_row_max_tiles() gives the tile count (0: this
  // plan cannot).  Greedy argmax then reads these candidates instead of the whole logits row.
  float2* row_max;
  // EPI_LSE only
  const int32_t* lse_targets;
  float* lse_target_out;
  // EPI_QKV only
  QkvEpilogue qe;
  // Decode (K-slice) kernels with both activation planes: read W_frag with non-temporal loads.  For weights
  // that will not be read again before the caches have turned over (a block decoder's, used once per L_B
  // steps; any stack too large for the 256 MB cache) this keeps them from displacing what is re-read.
  // All problems of a launch share the setting.
  int stream_w = 0;
};
// bf16 weights W[N, K] (K % 32 == 0) re-ordered for the decode GEMM: tiles of 16 rows x 32 k,
// tile (i, j) at element offset (i * K/32 + j) * 512; inside a tile lane l (0..63) owns the 8
// consecutive elements W[16 i + (l & 15)][32 j + 8 (l >> 4) ...], i.e. exactly the B operand of
// one 16x16x32 MFMA, so a wavefront fetches a fragment as 1 KB of consecutive bytes.
// Rows past N (N rounded up to 16) are zero.
size_t gemm_packed_elems(int N, int K);
hipError_t gemm_pack_weights(const void* W, void* W_frag, int N, int K, hipStream_t s);
// Which kernel serves a group of up to two problems, and into how many equal K
// parts each EPI_PARTIAL problem is split (others: 1).  Depends on shapes only.
struct GemmPlan {
  int kind, kf, nt, mc;
  int splits[2];
  int uneven;    // 1: splits need not divide the K-slice count (the first slices % splits walk one slice more)
};
hipError_t gemm_plan(int dtype, const GemmProblem* probs, int n_probs, GemmPlan* plan);
// Whether the kernel this plan selects is one of the tiled MFMA kernels, which implement EPI_LSE and EPI_QKV.
bool gemm_has_lse_epilogue(const GemmPlan& plan);
// Number of candidate tiles the launch writes per row (0: this plan does not produce them).
int gemm_row_max_tiles(const GemmProblem& p, const GemmPlan& plan);
// Raises the dynamic-LDS limit of every GEMM kernel that needs it, for the current device.  Call once
// per model before the first launch_gemm (and before any stream capture).
hipError_t gemm_prepare_kernels();
// Up to two independent problems in one launch.
hipError_t launch_gemm(int dtype, const GemmProblem* probs, int n_probs, const GemmPlan& plan, hipStream_t s);

// A matrix [rows, ld] that may still be in pieces: value(row, col) =
// (bias ? bias[col] : 0) + sum over s < splits of base[s * stride + row * ld + col].
struct PartialSrc {
  const float* base;
  const float* bias;
  int splits;
  size_t stride;
};

// MLP hidden activation from the up-projection's partial sums:
// out[row, col] = gelu(value(row, col)) stored as a GEMM operand (hi / lo planes when out_lo_off).
// Can ride along an attention launch (extra workgroups) or run alone.
struct GeluJob {
  PartialSrc src;
  void* out;
  size_t out_lo_off;
  int rows, cols;      // rows == 0: no job
};
hipError_t launch_gelu_reduce(int dtype, const GeluJob& job, hipStream_t s);

// ------------------------------------------------------------------ attention
// Rotary tables: rope[pos * (rot/2) + t] = (cos, sin) of pos * 10000^(-2t/rot).
hipError_t launch_rope_table(float2* tab, int n_pos, int rot, hipStream_t s);
//
// Block decoder prefill, after the QKV GEMM: rotate q in place (float, inside qkv),
// rotate k, and store k, v into the block KV cache at position pos0 + m % n_new
// of sequence m / n_new.  Cache layout per layer: K [B][H][n_cap][d_h], V same.
// qkv may arrive as split-K partials (src.splits > 1 and/or src.bias): the rotated q is then
// written complete into plane 0 (src.base), which is what the attention kernels read.
hipError_t launch_rope_append(int dtype, const PartialSrc& src, void* Kc, void* Vc, const float2* rope,
                              int n_rows, int n_new, int pos0, int n_heads, int d_head, int rot,
                              int n_cap, const GeluJob& gelu, hipStream_t s);

// Block decoder decode step, fused: finish q, k, v of every (b, h) from the (possibly split-K)
// QKV output, rotate q and k at position n_old, append k, v to the cache at slot n_old, and
// attend the one query to cache rows [0, n_old].  out [B, D] storage dtype (out_lo_off != 0:
// also the bf16 remainder plane).  n_dev: when non-null, sequence b reads its own n_old from
// device memory (n_dev[b]): a captured graph stays valid while the caches grow, and the
// sequences of a batch may hold different numbers of blocks.  gelu: optional job
// done by extra workgroups of the same launch.  n_split > 1: the cached rows of every (b, h) are
// cut into n_split ranges, one workgroup each, merged by a second small launch through split_buf
// (float [batch * n_heads * n_split][d_head + 2]); attn_block_decode_splits() gives the count this
// library uses for a batch, head count and cache capacity (1 when there are 256 pairs or more).
hipError_t launch_attn_block_decode(int dtype, const PartialSrc& qkv, void* Kc, void* Vc, const float2* rope, int rot,
                                    void* out, size_t out_lo_off, int batch, int n_heads, int d_head, int n_old,
                                    const int* n_dev, int n_cap, const GeluJob& gelu, int n_split, float* split_buf,
                                    hipStream_t s);
int attn_block_decode_splits(int batch, int n_heads, int n_cap);

// Block decoder prefill: causal attention of n_q queries per (b, h); query i sees rows [0, i].
hipError_t launch_attn_block_prefill(int dtype, const float* qkv, const void* Kc, const void* Vc,
                                     void* out, size_t out_lo_off, int batch, int n_heads, int d_head, int n_q,
                                     int n_cap, hipStream_t s);

// Token decoder: `rows` new local positions pos0 .. pos0+rows-1 per sequence.
// Rotates q, k; appends k, v to the local cache [B][H][l_cap][d_h]; causal
// attention over local rows [0, pos0+i]; out [B*rows, D] storage dtype.
hipError_t launch_attn_local(int dtype, const PartialSrc& qkv, void* Kl, void* Vl, const float2* rope,
                             void* out, size_t out_lo_off, int batch, int n_heads, int d_head, int rot, int rows,
                             int pos0, int l_cap, const GeluJob& gelu, hipStream_t s);

}  // namespace bt
