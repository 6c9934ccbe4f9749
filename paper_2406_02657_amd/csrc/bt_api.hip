// C ABI of the library: argument checks, workspace layout, and the host-side
// sequencing of the generation step (Sec. 2.1, Fig. 1, App. C of the paper).
// Every step of the path runs in the HIP kernels declared in kernels.h; this
// file only decides which launch comes next.
#include "../../include/bt.h"
#include "kernels.h"

#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using namespace bt;

namespace {

constexpr int kDefaultPrefillRows = 16384;
constexpr int kMaxSplits = 16;
// Weight bytes the decode steps try to keep in the 256 MB cache from one step to the next; the rest of the
// cache is left to activations and partial sums.  cfg1: 170 MB of token-decoder layers stay, the 77 MB head
// is streamed (443.1 -> 430.9 us per step against keeping both).
constexpr size_t kResidentBytes = (size_t)200 << 20;
constexpr int kSkinnyRows = 256;     // GEMMs with at most this many rows may split K

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Why the last bt_create / bt_create_static of this thread failed (bt_last_error(NULL)).
thread_local std::string g_create_err;

// Workspace of bt_create_static: one array per GPU, held until the process ends.  In host code the
// array's name is only a stand-in for the symbol; the device address comes from
// hipGetSymbolAddress, once per device (static_workspace), and that pointer is what the model and
// every kernel use.
static __device__ __align__(256) unsigned char scratch[BT_STATIC_WORKSPACE_BYTES];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];            // device address of `scratch` on device i (null: not asked yet)
const bt_model* g_scratch_owner[kMaxDevices];   // the live model that uses it, if any

struct Layout {
  size_t blk_kv, loc_kv, rope, x, u1, u2, qkv, ao, hmid, part_o, part_d, part_u, ctx, hfin, logits, cand, cur, state, lens, fin, summands, attn_split, score_kv, score_logits, frag, total;
  size_t blk_layer_stride, loc_layer_stride;   // bytes between layers (K then V inside)
  size_t part_elems;                           // floats in each of part_o, part_d
  size_t qkv_elems, part_u_elems;              // floats in qkv (may hold split-K pieces) and part_u
  size_t score_target_cap = 0;                 // rows of a chunk whose targets fit the scoring buffer
  int m_rows, l_cap, n_pref, rope_len, esz;
};

int check_config(const bt_config& c, std::string* why) {
  auto bad = [&](const char* s) { if (why) *why = s; return (int)BT_ERR_ARG; };
  if (c.struct_size != (int32_t)sizeof(bt_config)) return bad("struct_size is not sizeof(bt_config) of this library");
  if (c.dtype != BT_F32 && c.dtype != BT_BF16) return bad("dtype must be BT_F32 or BT_BF16");
  if (c.vocab < 1 || c.block_len < 1 || c.d_model < 1 || c.n_heads < 1 || c.d_ff < 1) return bad("non-positive size");
  if (c.n_block_layers < 0 || c.n_token_layers < 0) return bad("negative layer count");
  if (c.max_batch < 1 || c.max_blocks < 1) return bad("max_batch and max_blocks must be >= 1");
  if (c.d_model % c.n_heads) return bad("d_model % n_heads != 0");
  const int dh = c.d_model / c.n_heads;
  if (dh != 32 && dh != 64 && dh != 128) return bad("d_head must be 32, 64 or 128");
  if (c.d_model % c.block_len) return bad("d_model % block_len != 0");
  if ((c.d_model / c.block_len) % 8) return bad("d_emb must be a multiple of 8");
  if (c.d_model > 4096) return bad("d_model > 4096");
  if (c.rotary_dims < 0 || (c.rotary_dims & 1) || c.rotary_dims > dh) return bad("rotary_dims must be even and <= d_head");
  if (c.prefix_len < 0 || (c.prefix_len == 0 && c.block_len != 1)) return bad("prefix_len == 0 needs block_len == 1");
  if (c.dtype == BT_BF16 && (c.d_model % 64 || c.d_ff % 64)) return bad("bf16 mode needs d_model, d_ff multiples of 64");
  if (c.d_ff % 8) return bad("d_ff must be a multiple of 8");
  if (c.prefill_rows < 0) return bad("prefill_rows < 0");
  if (c.act_split < 0 || c.act_split > 2) return bad("act_split must be 0, 1 or 2");
  if (c.use_graphs < 0 || c.use_graphs > 1) return bad("use_graphs must be 0 or 1");
  if (c.pad_id < 0 || c.pad_id >= c.vocab) return bad("pad_id outside the vocabulary");
  if (c.eos_id < -1 || c.eos_id >= c.vocab) return bad("eos_id must be -1 (none) or a vocabulary id");
  if (c.score_rows < 0) return bad("score_rows < 0");
  if (c.keep_logits < 0 || c.keep_logits > 1) return bad("keep_logits must be 0 or 1");
  if (c.token_mix != BT_MIX_PREFIX && c.token_mix != BT_MIX_SUM) return bad("token_mix must be BT_MIX_PREFIX or BT_MIX_SUM");
  if (c.token_mix == BT_MIX_SUM && (c.prefix_len != 1 || c.score_rows != 0 || c.n_token_layers < 1))
    return bad("BT_MIX_SUM needs prefix_len == 1, score_rows == 0 and at least one token-decoder layer");
  if (!(c.ln_eps >= 0.f)) return bad("ln_eps < 0");
  const int l_cap = (c.prefix_len > 0 ? c.prefix_len : 1) + c.block_len;
  if ((size_t)(2 * l_cap + 2) * dh * sizeof(float) > 60 * 1024) return bad("prefix_len + block_len too large for the local-attention kernel");
  return BT_OK;
}

void make_layout(const bt_config& c, Layout& L) {
  const size_t D = c.d_model, F = c.d_ff, B = c.max_batch, H = c.n_heads, dh = D / H;
  L.esz = c.dtype == BT_BF16 ? 2 : 4;
  L.n_pref = c.prefix_len > 0 ? c.prefix_len : 1;
  L.l_cap = L.n_pref + c.block_len;
  L.rope_len = c.max_blocks > L.l_cap ? c.max_blocks : L.l_cap;
  size_t pr = c.prefill_rows > 0 ? c.prefill_rows : kDefaultPrefillRows;
  // rows one sequence needs at once: its blocks (prefill), times the token-decoder rows per block when
  // the model also scores whole sequences
  const size_t per_seq = (size_t)c.max_blocks * (c.score_rows > 0 ? L.n_pref + c.block_len - 1 : 1);
  if (pr < per_seq) pr = per_seq;
  if (pr > B * per_seq) pr = B * per_seq;
  size_t m_rows = pr;
  if (m_rows < B * L.n_pref) m_rows = B * L.n_pref;
  L.m_rows = (int)m_rows;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  L.blk_layer_stride = align_up(2 * B * H * c.max_blocks * dh * L.esz);
  L.blk_kv = take(L.blk_layer_stride * c.n_block_layers);
  L.loc_layer_stride = align_up(2 * B * H * L.l_cap * dh * L.esz);
  L.loc_kv = take(L.loc_layer_stride * c.n_token_layers);
  L.rope = take((size_t)L.rope_len * (c.rotary_dims / 2 + 1) * sizeof(float2));
  L.x = take(m_rows * D * 4);
  L.u1 = take(m_rows * D * 4);          // sized for float so that fp32 mode fits
  L.u2 = take(m_rows * D * 4);
  // Skinny (decode) GEMMs may leave up to K/64 split-K pieces for their consumers.
  const size_t skinny = m_rows < (size_t)kSkinnyRows ? m_rows : (size_t)kSkinnyRows;
  const size_t sD = D / 64 > 0 ? D / 64 : 1, sF = F / 64 > 0 ? F / 64 : 1;
  L.qkv_elems = m_rows * 3 * D;
  if (L.qkv_elems < sD * skinny * 3 * D) L.qkv_elems = sD * skinny * 3 * D;
  L.qkv = take(L.qkv_elems * 4);
  L.ao = take(m_rows * D * 4);
  L.hmid = take(m_rows * F * 4);
  L.part_elems = m_rows * D;
  const size_t sMax = sF > (size_t)kMaxSplits ? sF : (size_t)kMaxSplits;
  if (L.part_elems < sMax * skinny * D) L.part_elems = sMax * skinny * D;
  L.part_o = take(L.part_elems * 4);
  L.part_d = take(L.part_elems * 4);
  L.part_u_elems = sD * skinny * F;
  L.part_u = take(L.part_u_elems * 4);
  L.ctx = take(B * D * 4);
  L.hfin = take(B * D * 4);
  L.logits = take(B * (size_t)c.vocab * 4);
  L.cand = take(B * (size_t)((c.vocab + 63) / 64) * sizeof(float2));   // per-tile argmax candidates of the LM head
  L.cur = take(B * c.block_len * 4);
  L.state = take(B * 4);       // cached blocks per sequence (device-side counters)
  L.lens = take(B * 4);        // prompt lengths of the last prefill
  L.fin = take(B * 4);         // per sequence: has emitted eos_id
  // block-decoder decode attention at small batches: the ranges' partial results (at most 16 ranges of 255 pairs)
  L.attn_split = take((size_t)16 * 256 * (dh + 2) * 4);
  // summation token decoder: the L_B vectors the context embedding was projected to, per sequence
  L.summands = take(c.token_mix == BT_MIX_SUM ? B * c.block_len * D * 4 : 0);
  // teacher-forced scoring (score_rows > 0): the local KV of every block scored in one chunk (one
  // layer's worth, re-used by all layers) and the logits of score_rows rows at a time
  L.score_kv = L.score_logits = off;
  if (c.score_rows > 0) {
    const size_t lq = L.n_pref + c.block_len - 1;
    L.score_kv = take(2 * (m_rows / lq + 1) * H * L.l_cap * dh * L.esz);
    L.score_logits = take((size_t)c.score_rows * c.vocab * 4);
    // the same buffer, when the head's GEMM keeps the logits to itself: stats, target logits, then targets
    const size_t fixed = (size_t)c.score_rows * ((c.vocab + 63) / 64) * 8 + (size_t)c.score_rows * 4;
    L.score_target_cap = (size_t)c.score_rows * c.vocab * 4 > fixed ? ((size_t)c.score_rows * c.vocab * 4 - fixed) / 4 : 0;
  }
  // bf16 mode: a second copy of every GEMM weight in MFMA fragment order, read by the decode GEMMs
  L.frag = off;
  if (c.dtype == BT_BF16) {
    const size_t per_layer = align_up(gemm_packed_elems(3 * (int)D, (int)D) * 2) + align_up(gemm_packed_elems((int)D, (int)D) * 2) +
                             align_up(gemm_packed_elems((int)F, (int)D) * 2) + align_up(gemm_packed_elems((int)D, (int)F) * 2);
    take(per_layer * (c.n_block_layers + c.n_token_layers));
    take(gemm_packed_elems(c.vocab, (int)D) * 2);
    if (c.prefix_len > 0) take(gemm_packed_elems((c.token_mix == BT_MIX_SUM ? c.block_len : c.prefix_len) * (int)D, (int)D) * 2);
  }
  L.total = off;
}

}  // namespace

struct bt_model {
  bt_config cfg;
  bt_weights w;
  std::vector<bt_layer_weights> blk, tok;
  // bf16 mode: the GEMM weights once more, in MFMA fragment order (inside the workspace)
  struct FragLayer { const void *qkv, *o, *up, *down; };
  std::vector<FragLayer> blk_frag, tok_frag;
  const void *head_frag, *prefix_frag;
  Layout L;
  char* ws;
  hipStream_t stream;
  int batch, n_blocks, r;          // n_blocks: cached blocks of the longest sequence
  int64_t blocks_sum;              // cached blocks summed over the batch
  bool have_context, stepped;
  bt_stats st;
  bool profile;
  std::vector<hipEvent_t> ev;      // pairs (start, stop)
  std::vector<int> ev_tag;         // per pair: 0 = block-decoder decode attention, 1 = decode-step GEMM
  size_t ev_used;
  std::string err;
  struct StepGraph { hipGraphExec_t exec = nullptr; int seen = 0; };
  std::vector<StepGraph> graphs;   // one per step kind: r = 0..L_B-1 without, [L_B] with the block decoder
  bool graphs_ok;
  int64_t graph_launches;
  int graph_captures;
  int static_dev = -1;             // >= 0: the workspace is the static array of this device (bt_create_static)
  // Decode GEMMs read weights with non-temporal loads unless they are to stay in the 256 MB cache until the
  // next step reads them again.  What a step re-reads (the token decoder, the LM head, and the block decoder
  // when L_B = 1) is kept, in execution order and a whole stack at a time, while it fits kResidentBytes; the
  // rest, and a block decoder that runs once per L_B > 1 steps, is streamed past the cache.
  int resident_block_layers = 0, resident_token_layers = 0, resident_head = 0;

  template <class T> T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }
};

namespace {

int fail(bt_model* m, int code, const std::string& msg) {
  if (m) m->err = msg;
  return code;
}

#define BT_HIP(m, expr)                                                                  \
  do {                                                                                   \
    hipError_t e_ = (expr);                                                              \
    if (e_ != hipSuccess)                                                                \
      return fail((m), BT_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));   \
  } while (0)

void drop_graphs(bt_model* m) {
  for (auto& g : m->graphs) {
    if (g.exec) (void)hipGraphExecDestroy(g.exec);
    g.exec = nullptr;
    g.seen = 0;
  }
}

// Profiling: a pair of HIP events around one launch, tagged by kind (bt_set_profile).
int prof_begin(bt_model* m, int tag) {
  if (m->ev_used + 2 > m->ev.size()) {
    hipEvent_t n0, n1;
    BT_HIP(m, hipEventCreate(&n0));
    BT_HIP(m, hipEventCreate(&n1));
    m->ev.push_back(n0);
    m->ev.push_back(n1);
    m->ev_tag.push_back(tag);
  }
  m->ev_tag[m->ev_used / 2] = tag;
  BT_HIP(m, hipEventRecord(m->ev[m->ev_used], m->stream));
  return BT_OK;
}
int prof_end(bt_model* m) {
  BT_HIP(m, hipEventRecord(m->ev[m->ev_used + 1], m->stream));
  m->ev_used += 2;
  return BT_OK;
}

enum Mode { MODE_BLOCK_PREFILL, MODE_BLOCK_DECODE, MODE_TOKEN };

struct StackArgs {
  Mode mode;
  int M;           // rows in the residual stream
  int batch;       // sequences in this call
  int b0;          // first sequence (cache offset)
  int rows;        // rows per sequence (prefill: N_p; decode: 1; token: P or 1)
  int pos0;        // first position of the new rows
  // Optional: the first LayerNorm launch of the stack reads its rows from an embedding table
  // (row i = table[ids[i * stride + off]]) and writes them into the residual stream.
  const void* emb_table = nullptr;
  const int32_t* emb_ids = nullptr;
  int emb_stride = 0, emb_off = 0;
  // Optional: the stack's final LayerNorm launch adds one to counter_inc[i] for its row i.
  int* counter_inc = nullptr;
  // Optional: the final LayerNorm's row i is i * in_mul + fin_off_dev[i] - 1 (device memory).
  const int* fin_off_dev = nullptr;
  // Optional: where the final LayerNorm's remainder plane goes (elements after its output; 0: the default).
  size_t fin_lo_off = 0;
  // Optional (summation token decoder): the stack's first LayerNorm launch adds add[i * add_stride ...] to
  // row i (and, without emb_table, takes that vector as the row).
  const float* add = nullptr;
  int add_stride = 0;
  // Optional (MODE_TOKEN): local K (then V at +loc_half bytes) of `batch` sequences, shared by all layers.
  char* loc_base = nullptr;
  size_t loc_half = 0;
};

// Final LayerNorm of a stack on row (i*in_mul + in_off) of x, for i < n.
int final_ln(bt_model* m, const StackArgs& a, const float* pendO, const float* biasO, int sO,
             const float* pendD, const float* biasD, int sD, const void* g, const void* b,
             void* out, int out_f32, int n, int in_mul, int in_off) {
  ResidLnArgs r{};
  r.lo_off = (!out_f32 && m->cfg.dtype == BT_BF16 && m->cfg.act_split >= 1)
                 ? (a.fin_lo_off ? a.fin_lo_off : (size_t)m->cfg.max_batch * m->cfg.d_model) : 0;
  r.x = m->at<float>(m->L.x);
  r.partA = pendO; r.biasA = biasO; r.splitsA = sO;
  r.partB = pendD; r.biasB = biasD; r.splitsB = sD;
  r.part_stride = (size_t)a.M * m->cfg.d_model;
  r.g1 = (const float*)g; r.b1 = (const float*)b; r.u1 = out; r.u1_f32 = out_f32;
  r.g2 = nullptr; r.b2 = nullptr; r.u2 = nullptr;
  r.n_rows = n; r.D = m->cfg.d_model; r.in_mul = in_mul; r.in_off = in_off; r.write_x = 0;
  r.eps = m->cfg.ln_eps;
  r.counter_inc = a.counter_inc;
  BT_HIP(m, launch_resid_ln(m->cfg.dtype, r, m->stream, a.fin_off_dev));
  return BT_OK;
}

// Runs n_layers decoder layers over x [M, D] and the stack's final LayerNorm.
int run_stack(bt_model* m, const bt_layer_weights* lw, int n_layers, const StackArgs& a,
              const void* fin_g, const void* fin_b, void* fin_out, int fin_f32, int fin_n, int fin_mul, int fin_off) {
  const bt_config& c = m->cfg;
  const Layout& L = m->L;
  const int D = c.d_model, F = c.d_ff, H = c.n_heads, dh = D / H, dt = c.dtype;
  float* x = m->at<float>(L.x);
  void* u1 = m->at<void>(L.u1);
  void* u2 = m->at<void>(L.u2);
  float* qkv = m->at<float>(L.qkv);
  void* ao = m->at<void>(L.ao);
  void* hmid = m->at<void>(L.hmid);
  float* part_o = m->at<float>(L.part_o);
  float* part_d = m->at<float>(L.part_d);
  float* part_u = m->at<float>(L.part_u);
  const float2* rope = m->at<float2>(L.rope);
  hipStream_t s = m->stream;
  const int M = a.M;
  const bt_model::FragLayer* fw = lw == m->blk.data() ? m->blk_frag.data() : m->tok_frag.data();
  if (n_layers == 0)
    return final_ln(m, a, nullptr, nullptr, 0, nullptr, nullptr, 0, fin_g, fin_b, fin_out, fin_f32, fin_n, fin_mul, fin_off);

  // bf16 mode: activations that feed GEMMs are kept as hi + remainder planes (see bt.h, act_split)
  const bool split = dt == BT_BF16 && (c.act_split == 2 || (c.act_split == 1 && a.mode != MODE_BLOCK_PREFILL));
  const size_t loD = split ? (size_t)L.m_rows * D : 0, loF = split ? (size_t)L.m_rows * F : 0;
  auto lo = [&](const void* p, size_t off) -> const void* { return off ? (const char*)p + off * 2 : nullptr; };
  // Skinny bf16 GEMMs (decode steps) hand raw split-K partial sums to their consumers, which add
  // bias / GELU / rotary; large or fp32 GEMMs finish their own epilogue.
  const bool pieces = dt == BT_BF16 && M <= kSkinnyRows;
  const void* a_up = c.parallel_residual ? u2 : u1;
  GemmProblem pq{u1, nullptr, nullptr, qkv, M, 3 * D, D, D, 3 * D, pieces ? EPI_PARTIAL : EPI_F32, lo(u1, loD), 0};
  GemmProblem pu{a_up, nullptr, nullptr, pieces ? (void*)part_u : hmid, M, F, D, D, F, pieces ? EPI_PARTIAL : EPI_GELU,
                 lo(a_up, loD), loF};
  GemmProblem po{ao, nullptr, nullptr, part_o, M, D, D, D, D, EPI_PARTIAL, lo(ao, loD), 0};
  GemmProblem pd{hmid, nullptr, nullptr, part_d, M, D, F, F, D, EPI_PARTIAL, lo(hmid, loF), 0};
  const int n_resident = (a.mode == MODE_TOKEN) ? m->resident_token_layers : m->resident_block_layers;
  GemmPlan plan_in{}, plan_out{}, plan_q{}, plan_u{}, plan_o{}, plan_d{};
  int sQ, sU, sO, sD;
  if (c.parallel_residual) {
    GemmProblem gi[2] = {pq, pu}, go[2] = {po, pd};
    BT_HIP(m, gemm_plan(dt, gi, 2, &plan_in));
    BT_HIP(m, gemm_plan(dt, go, 2, &plan_out));
    sQ = plan_in.splits[0]; sU = plan_in.splits[1];
    sO = plan_out.splits[0]; sD = plan_out.splits[1];
  } else {
    BT_HIP(m, gemm_plan(dt, &pq, 1, &plan_q));
    BT_HIP(m, gemm_plan(dt, &pu, 1, &plan_u));
    BT_HIP(m, gemm_plan(dt, &po, 1, &plan_o));
    BT_HIP(m, gemm_plan(dt, &pd, 1, &plan_d));
    sQ = plan_q.splits[0]; sU = plan_u.splits[0]; sO = plan_o.splits[0]; sD = plan_d.splits[0];
  }
  if ((size_t)sO * M * D > L.part_elems || (size_t)sD * M * D > L.part_elems ||
      (size_t)sQ * M * 3 * D > L.qkv_elems || (pieces && (size_t)sU * M * F > L.part_u_elems))
    return fail(m, BT_ERR_CAPACITY, "split-K partial buffer too small");

  // Prefill with the tiled MFMA kernels: rotary and the KV append ride in the QKV GEMM's epilogue
  const bool qkv_fused = a.mode == MODE_BLOCK_PREFILL && !pieces && dt == BT_BF16 && c.parallel_residual &&
                         gemm_has_lse_epilogue(plan_in) && gemm_qkv_epilogue_ok(D, dh, c.rotary_dims);
  auto qkv_epilogue = [&](int l, GemmProblem& p) {
    char* base = m->ws + L.blk_kv + (size_t)l * L.blk_layer_stride;
    const size_t half = (size_t)c.max_batch * H * c.max_blocks * dh * L.esz;
    const size_t seq = (size_t)a.b0 * H * c.max_blocks * dh * L.esz;
    p.epi = EPI_QKV;
    p.qe = QkvEpilogue{rope, base + seq, base + half + seq, a.rows, a.pos0, H, dh, c.rotary_dims, c.max_blocks};
  };
  auto ln = [&](const float* pO, const float* bO, int nO, const float* pD, const float* bD, int nD,
                const void* g1, const void* b1, const void* g2, const void* b2) -> int {
    ResidLnArgs r{};
    r.x = x;
    r.partA = pO; r.biasA = bO; r.splitsA = nO;
    r.partB = pD; r.biasB = bD; r.splitsB = nD;
    r.part_stride = (size_t)M * D;
    r.g1 = (const float*)g1; r.b1 = (const float*)b1; r.u1 = u1; r.u1_f32 = 0;
    r.g2 = (const float*)g2; r.b2 = (const float*)b2; r.u2 = u2;
    r.n_rows = M; r.D = D; r.in_mul = 1; r.in_off = 0; r.write_x = (pO || pD) ? 1 : 0;
    r.eps = c.ln_eps;
    r.lo_off = loD;
    if (!pO && !pD && a.emb_table) {        // first launch of the stack: rows come from the table
      r.emb_table = a.emb_table; r.emb_ids = a.emb_ids; r.emb_stride = a.emb_stride; r.emb_off = a.emb_off;
      r.write_x = 1;
    }
    if (!pO && !pD && a.add) {              // ... plus (or only) the summand of this local position
      r.add = a.add; r.add_stride = a.add_stride;
      r.write_x = 1;
    }
    BT_HIP(m, launch_resid_ln(dt, r, s));
    return BT_OK;
  };
  // attention of layer l; `gelu` (may be empty) rides along as extra workgroups of the local
  // attention or of the rotary/append launch
  auto attention = [&](int l, const GeluJob& gelu) -> int {
    const PartialSrc qsrc{qkv, pieces ? (const float*)lw[l].b_qkv : nullptr, sQ, (size_t)M * 3 * D};
    if (a.mode == MODE_TOKEN) {
      char* base = a.loc_base ? a.loc_base : m->ws + L.loc_kv + (size_t)l * L.loc_layer_stride;
      const size_t half = a.loc_base ? a.loc_half : (size_t)c.max_batch * H * L.l_cap * dh * L.esz;
      BT_HIP(m, launch_attn_local(dt, qsrc, base, base + half, rope, ao, loD, a.batch, H, dh, c.rotary_dims,
                                  a.rows, a.pos0, L.l_cap, gelu, s));
      return BT_OK;
    }
    char* base = m->ws + L.blk_kv + (size_t)l * L.blk_layer_stride;
    const size_t half = (size_t)c.max_batch * H * c.max_blocks * dh * L.esz;
    const size_t seq = (size_t)a.b0 * H * c.max_blocks * dh * L.esz;
    char* Kc = base + seq;
    char* Vc = base + half + seq;
    if (a.mode == MODE_BLOCK_PREFILL) {
      if (!qkv_fused)        // else the QKV GEMM's epilogue has rotated q and k and filled the cache
        BT_HIP(m, launch_rope_append(dt, qsrc, Kc, Vc, rope, M, a.rows, a.pos0, H, dh, c.rotary_dims,
                                     c.max_blocks, gelu, s));
      BT_HIP(m, launch_attn_block_prefill(dt, qkv, Kc, Vc, ao, loD, a.batch, H, dh, a.rows, c.max_blocks, s));
    } else {
      const int n_old = a.pos0;
      int prc;
      if (m->profile && (prc = prof_begin(m, 0))) return prc;
      BT_HIP(m, launch_attn_block_decode(dt, qsrc, Kc, Vc, rope, c.rotary_dims, ao, loD, a.batch, H, dh, n_old,
                                         m->at<int>(L.state), c.max_blocks, gelu,
                                         attn_block_decode_splits(a.batch, H, c.max_blocks), m->at<float>(L.attn_split), s));
      if (m->profile) {
        if ((prc = prof_end(m))) return prc;
        m->st.attn_block_launches += 1;
        m->st.attn_block_bytes += (int64_t)2 * (m->blocks_sum + a.batch) * D * L.esz;
      }
    }
    return BT_OK;
  };
  auto gelu_job = [&](int l) {
    GeluJob j{};
    if (pieces) {
      j.src = PartialSrc{part_u, (const float*)lw[l].b_up, sU, (size_t)M * F};
      j.out = hmid; j.out_lo_off = loF; j.rows = M; j.cols = F;
    }
    return j;
  };
  const GeluJob no_job{};

  int rc;
  if (c.parallel_residual) {
    if ((rc = ln(nullptr, nullptr, 0, nullptr, nullptr, 0, lw[0].ln1_g, lw[0].ln1_b, lw[0].ln2_g, lw[0].ln2_b))) return rc;
    for (int l = 0; l < n_layers; ++l) {
      GemmProblem p[2] = {pq, pu};
      p[0].W = lw[l].W_qkv; p[1].W = lw[l].W_up;
      p[0].stream_w = p[1].stream_w = l >= n_resident;
      p[0].W_frag = fw[l].qkv; p[1].W_frag = fw[l].up;
      if (!pieces) { p[0].bias = (const float*)lw[l].b_qkv; p[1].bias = (const float*)lw[l].b_up; }
      if (qkv_fused) qkv_epilogue(l, p[0]);
      const bool prof_gemm = m->profile && pieces, prof_tiled = m->profile && !pieces;
      if (m->profile && (rc = prof_begin(m, pieces ? 1 : 2))) return rc;
      BT_HIP(m, launch_gemm(dt, p, 2, plan_in, s));
      if (m->profile && (rc = prof_end(m))) return rc;
      if (prof_gemm) {
        m->st.gemm_decode_launches += 1;
        m->st.gemm_decode_bytes += (int64_t)(3 * D + F) * D * L.esz;
      }
      if (prof_tiled) {
        m->st.gemm_tiled_launches += 1;
        m->st.gemm_tiled_flops += (int64_t)2 * M * (3 * D + F) * D;
      }
      if ((rc = attention(l, gelu_job(l)))) return rc;
      p[0] = po; p[0].W = lw[l].W_o; p[0].W_frag = fw[l].o;
      p[0].stream_w = l >= n_resident;
      p[1] = pd; p[1].W = lw[l].W_down; p[1].W_frag = fw[l].down;
      p[1].stream_w = l >= n_resident;
      if (m->profile && (rc = prof_begin(m, pieces ? 1 : 2))) return rc;
      BT_HIP(m, launch_gemm(dt, p, 2, plan_out, s));
      if (m->profile && (rc = prof_end(m))) return rc;
      if (prof_gemm) {
        m->st.gemm_decode_launches += 1;
        m->st.gemm_decode_bytes += (int64_t)(D + F) * D * L.esz;
      }
      if (prof_tiled) {
        m->st.gemm_tiled_launches += 1;
        m->st.gemm_tiled_flops += (int64_t)2 * M * (D + F) * D;
      }
      if (l + 1 < n_layers) {
        if ((rc = ln(part_o, (const float*)lw[l].b_o, sO, part_d, (const float*)lw[l].b_down, sD,
                     lw[l + 1].ln1_g, lw[l + 1].ln1_b, lw[l + 1].ln2_g, lw[l + 1].ln2_b))) return rc;
      } else {
        return final_ln(m, a, part_o, (const float*)lw[l].b_o, sO, part_d, (const float*)lw[l].b_down, sD,
                        fin_g, fin_b, fin_out, fin_f32, fin_n, fin_mul, fin_off);
      }
    }
  } else {
    if ((rc = ln(nullptr, nullptr, 0, nullptr, nullptr, 0, lw[0].ln1_g, lw[0].ln1_b, nullptr, nullptr))) return rc;
    for (int l = 0; l < n_layers; ++l) {
      pq.stream_w = po.stream_w = pu.stream_w = pd.stream_w = l >= n_resident;
      GemmProblem p = pq;
      p.W = lw[l].W_qkv; p.W_frag = fw[l].qkv;
      if (!pieces) p.bias = (const float*)lw[l].b_qkv;
      BT_HIP(m, launch_gemm(dt, &p, 1, plan_q, s));
      if ((rc = attention(l, no_job))) return rc;
      p = po; p.W = lw[l].W_o; p.W_frag = fw[l].o;
      BT_HIP(m, launch_gemm(dt, &p, 1, plan_o, s));
      if ((rc = ln(part_o, (const float*)lw[l].b_o, sO, nullptr, nullptr, 0, lw[l].ln2_g, lw[l].ln2_b, nullptr, nullptr))) return rc;
      p = pu; p.W = lw[l].W_up; p.W_frag = fw[l].up;
      if (!pieces) p.bias = (const float*)lw[l].b_up;
      BT_HIP(m, launch_gemm(dt, &p, 1, plan_u, s));
      BT_HIP(m, launch_gelu_reduce(dt, gelu_job(l), s));
      p = pd; p.W = lw[l].W_down; p.W_frag = fw[l].down;
      BT_HIP(m, launch_gemm(dt, &p, 1, plan_d, s));
      if (l + 1 < n_layers) {
        if ((rc = ln(nullptr, nullptr, 0, part_d, (const float*)lw[l].b_down, sD, lw[l + 1].ln1_g, lw[l + 1].ln1_b, nullptr, nullptr))) return rc;
      } else {
        return final_ln(m, a, nullptr, nullptr, 0, part_d, (const float*)lw[l].b_down, sD,
                        fin_g, fin_b, fin_out, fin_f32, fin_n, fin_mul, fin_off);
      }
    }
  }
  return BT_OK;
}

}  // namespace

extern "C" {

int bt_workspace_bytes(const bt_config* cfg, size_t* bytes) {
  if (!cfg || !bytes) return BT_ERR_ARG;
  int rc = check_config(*cfg, nullptr);
  if (rc) return rc;
  Layout L;
  make_layout(*cfg, L);
  *bytes = L.total;
  return BT_OK;
}

// Everything bt_create and bt_create_static share.  Calls no HIP allocation routine: the model
// lives in host memory, all device memory is the caller's (or the static array).
static int create_impl(const bt_config* cfg, const bt_weights* w, void* workspace_dev, size_t workspace_bytes,
                       void* hip_stream, bt_model** out) {
  auto bad = [](int code, const char* why) { g_create_err = why; return code; };
  if (!cfg || !w || !out) return bad(BT_ERR_ARG, "null argument");
  *out = nullptr;
  if (!workspace_dev || ((uintptr_t)workspace_dev & 255)) return bad(BT_ERR_ARG, "workspace is null or not 256-byte aligned");
  int rc = check_config(*cfg, &g_create_err);
  if (rc) return rc;
  const bool need_tok_table = cfg->block_len > 1;
  if (!w->E_emb || !w->W_head || !w->blk_lnf_g || !w->blk_lnf_b || !w->tok_lnf_g || !w->tok_lnf_b) return bad(BT_ERR_ARG, "a weight pointer is null");
  if (need_tok_table && !w->E_tok) return bad(BT_ERR_ARG, "E_tok is null");
  if (cfg->prefix_len > 0 && (!w->W_prefix || !w->b_prefix)) return bad(BT_ERR_ARG, "W_prefix or b_prefix is null");
  if ((cfg->n_block_layers > 0 && !w->block_layers) || (cfg->n_token_layers > 0 && !w->token_layers)) return bad(BT_ERR_ARG, "layer array is null");
  auto layer_ok = [](const bt_layer_weights& l) {
    return l.ln1_g && l.ln1_b && l.W_qkv && l.b_qkv && l.W_o && l.b_o && l.ln2_g && l.ln2_b && l.W_up && l.b_up &&
           l.W_down && l.b_down;
  };
  for (int i = 0; i < cfg->n_block_layers; ++i) if (!layer_ok(w->block_layers[i])) return bad(BT_ERR_ARG, "a block-decoder layer pointer is null");
  for (int i = 0; i < cfg->n_token_layers; ++i) if (!layer_ok(w->token_layers[i])) return bad(BT_ERR_ARG, "a token-decoder layer pointer is null");
  Layout L;
  make_layout(*cfg, L);
  if (workspace_bytes < L.total) return bad(BT_ERR_CAPACITY, "workspace smaller than bt_workspace_bytes");

  bt_model* m = new (std::nothrow) bt_model();
  if (!m) return bad(BT_ERR_ARG, "out of host memory");
  m->cfg = *cfg;
  {
    const size_t esz = cfg->dtype == BT_BF16 ? 2 : 4, D = (size_t)cfg->d_model;
    const size_t layer = (4 * D * D + 2 * D * (size_t)cfg->d_ff) * esz, head = (size_t)cfg->vocab * D * esz;
    size_t room = kResidentBytes;
    // a stack is kept whole or not at all: with half of cfg3's token decoder kept (8 of 16 layers, 201 MB) a step took
    // 886.7 us against 870.5 us with all of it streamed
    auto keep = [&](int n_layers) { const int k = (size_t)n_layers * layer <= room ? n_layers : 0; room -= (size_t)k * layer; return k; };
    if (cfg->block_len == 1) m->resident_block_layers = keep(cfg->n_block_layers);
    m->resident_token_layers = (cfg->block_len > 1 || m->resident_block_layers == cfg->n_block_layers) ? keep(cfg->n_token_layers) : 0;
    m->resident_head = m->resident_token_layers == cfg->n_token_layers && head <= room;
  }
  m->w = *w;
  m->blk.assign(w->block_layers, w->block_layers + cfg->n_block_layers);
  m->tok.assign(w->token_layers, w->token_layers + cfg->n_token_layers);
  m->w.block_layers = m->blk.data();
  m->w.token_layers = m->tok.data();
  m->L = L;
  m->ws = reinterpret_cast<char*>(workspace_dev);
  m->stream = reinterpret_cast<hipStream_t>(hip_stream);
  m->batch = 0; m->n_blocks = 0; m->blocks_sum = 0; m->r = 0;
  m->have_context = false; m->stepped = false;
  std::memset(&m->st, 0, sizeof(m->st));
  m->profile = false;
  m->ev_used = 0;
  m->graphs.assign(cfg->block_len + 1, bt_model::StepGraph());
  m->graphs_ok = true;
  m->graph_launches = 0;
  m->graph_captures = 0;
  if (cfg->use_graphs && !m->stream) {
    m->graphs_ok = false;
    m->err = "HIP graphs need a stream other than the default stream: decode steps are launched eagerly";
  }
  {
    const hipError_t pe = gemm_prepare_kernels();
    if (pe != hipSuccess) {
      (void)hipGetLastError();
      delete m;
      g_create_err = std::string("raising the LDS limit of the GEMM kernels failed: ") + hipGetErrorString(pe);
      return BT_ERR_HIP;
    }
  }

  m->blk_frag.assign(cfg->n_block_layers, bt_model::FragLayer{nullptr, nullptr, nullptr, nullptr});
  m->tok_frag.assign(cfg->n_token_layers, bt_model::FragLayer{nullptr, nullptr, nullptr, nullptr});
  m->head_frag = nullptr; m->prefix_frag = nullptr;
  if (cfg->dtype == BT_BF16) {
    const int D = cfg->d_model, F = cfg->d_ff;
    size_t off = L.frag;
    hipError_t e = hipSuccess;
    auto pack = [&](const void* W, int N, int K) -> const void* {
      void* dst = m->ws + off;
      off = align_up(off + gemm_packed_elems(N, K) * 2);
      if (e == hipSuccess) e = gemm_pack_weights(W, dst, N, K, m->stream);
      return dst;
    };
    auto pack_layers = [&](const std::vector<bt_layer_weights>& lw, std::vector<bt_model::FragLayer>& fw) {
      for (size_t i = 0; i < lw.size(); ++i) {
        fw[i].qkv = pack(lw[i].W_qkv, 3 * D, D);
        fw[i].o = pack(lw[i].W_o, D, D);
        fw[i].up = pack(lw[i].W_up, F, D);
        fw[i].down = pack(lw[i].W_down, D, F);
      }
    };
    pack_layers(m->blk, m->blk_frag);
    pack_layers(m->tok, m->tok_frag);
    m->head_frag = pack(w->W_head, cfg->vocab, D);
    if (cfg->prefix_len > 0)
      m->prefix_frag = pack(w->W_prefix, (cfg->token_mix == BT_MIX_SUM ? cfg->block_len : cfg->prefix_len) * D, D);
    if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
    if (e != hipSuccess || off > L.total) { delete m; return bad(BT_ERR_HIP, "re-ordering the weights failed"); }
  }

  // rotary table: (cos, sin) of pos * 10000^(-2t/rot), computed in double by a small kernel
  if (cfg->rotary_dims > 0) {
    hipError_t e = launch_rope_table(m->at<float2>(L.rope), L.rope_len, cfg->rotary_dims, m->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
    if (e != hipSuccess) { delete m; return bad(BT_ERR_HIP, "filling the rotary table failed"); }
  }
  *out = m;
  return BT_OK;
}

int bt_create(const bt_config* cfg, const bt_weights* w, void* workspace_dev, size_t workspace_bytes,
              void* hip_stream, bt_model** out) {
  return create_impl(cfg, w, workspace_dev, workspace_bytes, hip_stream, out);
}

int bt_create_static(const bt_config* cfg, const bt_weights* w, void* hip_stream, bt_model** out) {
  auto bad = [](int code, const char* why) { g_create_err = why; return code; };
  if (!cfg || !w || !out) return bad(BT_ERR_ARG, "null argument");
  *out = nullptr;
  int rc = check_config(*cfg, &g_create_err);
  if (rc) return rc;
  Layout L;
  make_layout(*cfg, L);
  if (L.total > (size_t)BT_STATIC_WORKSPACE_BYTES)
    return bad(BT_ERR_CAPACITY, "this config needs more workspace than BT_STATIC_WORKSPACE_BYTES: use bt_create with a workspace of bt_workspace_bytes");
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return bad(BT_ERR_HIP, "hipGetDevice failed"); }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    // once per device, with that device current: each GPU holds its own copy of the array at its own address
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) { (void)hipGetLastError(); return bad(BT_ERR_HIP, "hipGetSymbolAddress(scratch) failed"); }
    g_scratch_ptr[dev] = p;
  }
  if (g_scratch_owner[dev]) return bad(BT_ERR_STATE, "the static workspace of this GPU is in use by a live model: bt_destroy it first");
  bt_config c = *cfg;
  c.use_graphs = 0;                    // graph instantiation allocates; such a model never does
  rc = create_impl(&c, w, g_scratch_ptr[dev], BT_STATIC_WORKSPACE_BYTES, hip_stream, out);
  if (rc == BT_OK) {
    (*out)->static_dev = dev;
    g_scratch_owner[dev] = *out;
  }
  return rc;
}

// Prefill of `batch` prompts held in rows of `row_stride` ids.  lens_host null: every prompt has
// max_len ids; else sequence b has lens_host[b] <= max_len.  Every sequence is left-padded to
// whole blocks on its own, so all of them end on a block boundary and decode in lockstep; the
// shorter ones simply hold fewer cached blocks.
static int prefill_impl(bt_model* m, const int32_t* tokens_dev, int batch, int row_stride, int max_len,
                        const int32_t* lens_host) {
  const bt_config& c = m->cfg;
  const int n_p = (max_len + c.block_len - 1) / c.block_len;     // blocks of the longest prompt
  if (n_p > c.max_blocks) return fail(m, BT_ERR_CAPACITY, "prompt needs more block slots than max_blocks");
  const Layout& L = m->L;
  int per = L.m_rows / n_p;
  if (per < 1) return fail(m, BT_ERR_CAPACITY, "workspace rows < prompt blocks");
  int* seq_n = m->at<int>(L.state);
  int* seq_len = m->at<int>(L.lens);
  int64_t blocks_sum = (int64_t)batch * n_p;
  if (lens_host) {
    blocks_sum = 0;
    for (int b = 0; b < batch; ++b) blocks_sum += (lens_host[b] + c.block_len - 1) / c.block_len;
    BT_HIP(m, hipMemcpyAsync(seq_len, lens_host, (size_t)batch * sizeof(int32_t), hipMemcpyHostToDevice, m->stream));
    BT_HIP(m, hipStreamSynchronize(m->stream));                  // the caller's array is free again on return
    BT_HIP(m, launch_seq_blocks(seq_len, seq_n, c.block_len, batch, m->stream));
  } else {
    BT_HIP(m, launch_state_set(seq_len, max_len, batch, m->stream));
    BT_HIP(m, launch_state_set(seq_n, n_p, batch, m->stream));
  }
  BT_HIP(m, launch_state_set(m->at<int>(L.fin), 0, c.max_batch, m->stream));
  const bool ctx_f32 = c.prefix_len == 0;
  const size_t ctx_esz = ctx_f32 ? 4 : L.esz;
  for (int b0 = 0; b0 < batch; b0 += per) {
    const int bc = batch - b0 < per ? batch - b0 : per;
    BT_HIP(m, launch_embed_concat(c.dtype, m->w.E_emb, tokens_dev + (size_t)b0 * row_stride, m->at<float>(L.x),
                                  bc, n_p, c.block_len, c.d_model / c.block_len, row_stride, max_len, seq_len + b0,
                                  c.pad_id, m->stream));
    StackArgs a{MODE_BLOCK_PREFILL, bc * n_p, bc, b0, n_p, 0};
    a.fin_off_dev = seq_n + b0;             // the context embedding is the row of each sequence's own last block
    int rc = run_stack(m, m->blk.data(), c.n_block_layers, a, m->w.blk_lnf_g, m->w.blk_lnf_b,
                       m->ws + L.ctx + (size_t)b0 * c.d_model * ctx_esz, ctx_f32, bc, n_p, n_p - 1);
    if (rc) return rc;
  }
  if (batch != m->batch) drop_graphs(m);      // captured launches are sized for one batch
  m->batch = batch;
  m->n_blocks = n_p;
  m->blocks_sum = blocks_sum;
  m->r = 0;
  m->have_context = true;
  m->stepped = false;
  bt_stats& st = m->st;
  st.block_passes = n_p;
  st.token_passes = st.token_rows = st.block_kv_rows_read = st.block_kv_bytes_read = 0;
  st.local_kv_high_water = 0;
  return BT_OK;
}

int bt_prefill(bt_model* m, const int32_t* tokens_dev, int32_t batch, int32_t prompt_len) {
  if (!m) return BT_ERR_ARG;
  if (!tokens_dev) return fail(m, BT_ERR_ARG, "tokens_dev is null");
  if (batch < 1 || batch > m->cfg.max_batch) return fail(m, BT_ERR_ARG, "batch out of range");
  if (prompt_len < 1) return fail(m, BT_ERR_ARG, "prompt_len < 1");
  return prefill_impl(m, tokens_dev, batch, prompt_len, prompt_len, nullptr);
}

int bt_prefill_ragged(bt_model* m, const int32_t* tokens_dev, const int32_t* lens_host, int32_t batch, int32_t max_len) {
  if (!m) return BT_ERR_ARG;
  if (!tokens_dev || !lens_host) return fail(m, BT_ERR_ARG, "tokens_dev or lens_host is null");
  if (batch < 1 || batch > m->cfg.max_batch) return fail(m, BT_ERR_ARG, "batch out of range");
  if (max_len < 1) return fail(m, BT_ERR_ARG, "max_len < 1");
  int longest = 0;
  for (int b = 0; b < batch; ++b) {
    if (lens_host[b] < 1 || lens_host[b] > max_len) return fail(m, BT_ERR_ARG, "a prompt length lies outside [1, max_len]");
    if (lens_host[b] > longest) longest = lens_host[b];
  }
  return prefill_impl(m, tokens_dev, batch, max_len, longest, lens_host);
}

// Enqueue every launch of one decode step.  with_block: embed the finished block and run the
// block decoder first (r == 0 only).  ids_out: where argmax writes the ids besides the open
// block's buffer (null inside a captured graph, whose launches must not depend on the caller's
// output pointer).
static int enqueue_step(bt_model* m, int r, bool with_block, int32_t* ids_out) {
  const bt_config& c = m->cfg;
  const Layout& L = m->L;
  const int D = c.d_model, B = m->batch;
  hipStream_t s = m->stream;
  int32_t* cur = m->at<int32_t>(L.cur);
  float* x = m->at<float>(L.x);
  const bool ctx_f32 = c.prefix_len == 0;
  const size_t fin_lo = (c.dtype == BT_BF16 && c.act_split >= 1) ? (size_t)c.max_batch * D : 0;
  int rows, pos0;
  if (r == 0) {
    if (with_block) {
      BT_HIP(m, launch_embed_concat(c.dtype, m->w.E_emb, cur, x, B, 1, c.block_len, D / c.block_len, c.block_len,
                                    c.block_len, nullptr, c.pad_id, s));
      StackArgs a{MODE_BLOCK_DECODE, B, B, 0, 1, m->n_blocks};
      a.counter_inc = m->at<int>(L.state);     // the final LayerNorm launch counts the new block in
      int rc = run_stack(m, m->blk.data(), c.n_block_layers, a, m->w.blk_lnf_g, m->w.blk_lnf_b,
                         m->ws + L.ctx, ctx_f32, B, 1, 0);
      if (rc) return rc;
    }
    if (c.prefix_len > 0) {
      // prefix tokens go straight into the residual stream; the summands of the summation variant wait in
      // their own buffer and are added to the inputs position by position
      const bool sum = c.token_mix == BT_MIX_SUM;
      const int n_proj = sum ? c.block_len : c.prefix_len;
      GemmProblem p{m->ws + L.ctx, m->w.W_prefix, (const float*)m->w.b_prefix, sum ? m->at<float>(L.summands) : x, B, n_proj * D, D, D,
                    n_proj * D, EPI_F32, fin_lo ? m->ws + L.ctx + fin_lo * 2 : nullptr, 0, m->prefix_frag};
      p.stream_w = 1;                    // used once per block
      GemmPlan pl{};
      BT_HIP(m, gemm_plan(c.dtype, &p, 1, &pl));
      BT_HIP(m, launch_gemm(c.dtype, &p, 1, pl, s));
    } else {
      BT_HIP(m, launch_copy16(x, m->ws + L.ctx, (size_t)B * D * 4, s));
    }
    rows = L.n_pref;
    pos0 = 0;
  } else {
    // the token's embedding row is read by the first LayerNorm launch of the stack; without
    // layers there is no such launch
    if (c.n_token_layers == 0) BT_HIP(m, launch_token_embed(c.dtype, m->w.E_tok, cur, x, B, c.block_len, r - 1, D, s));
    rows = 1;
    pos0 = L.n_pref + r - 1;
  }
  StackArgs a{MODE_TOKEN, B * rows, B, 0, rows, pos0};
  if (r != 0 && c.n_token_layers > 0) { a.emb_table = m->w.E_tok; a.emb_ids = cur; a.emb_stride = c.block_len; a.emb_off = r - 1; }
  if (c.token_mix == BT_MIX_SUM) { a.add = m->at<float>(L.summands) + (size_t)r * D; a.add_stride = c.block_len * D; }
  int rc = run_stack(m, m->tok.data(), c.n_token_layers, a, m->w.tok_lnf_g, m->w.tok_lnf_b,
                     m->ws + L.hfin, 0, B, rows, rows - 1);
  if (rc) return rc;
  GemmProblem p{m->ws + L.hfin, m->w.W_head, nullptr, m->ws + L.logits, B, c.vocab, D, D, c.vocab, EPI_F32,
                fin_lo ? m->ws + L.hfin + fin_lo * 2 : nullptr, 0, m->head_frag};
  p.stream_w = !m->resident_head;
  GemmPlan pl{};
  BT_HIP(m, gemm_plan(c.dtype, &p, 1, &pl));
  // Greedy argmax: where the head's kernel can, it leaves per-tile (max, column) candidates per row
  // and a small kernel picks among them; otherwise one workgroup per row scans the logits.
  const int cand_tiles = gemm_row_max_tiles(p, pl);
  if (cand_tiles > 0) {
    p.row_max = m->at<float2>(L.cand);
    if (!c.keep_logits) p.out = nullptr;      // the head's kernel leaves the candidates only
  }
  BT_HIP(m, launch_gemm(c.dtype, &p, 1, pl, s));
  if (cand_tiles > 0)
    BT_HIP(m, launch_argmax_candidates(m->at<float2>(L.cand), cand_tiles, B, c.vocab, ids_out, cur, c.block_len, r, c.eos_id,
                                       m->at<int32_t>(L.fin), s));
  else
    BT_HIP(m, launch_argmax(m->at<float>(L.logits), B, c.vocab, ids_out, cur, c.block_len, r, c.eos_id,
                            m->at<int32_t>(L.fin), s));
  return BT_OK;
}

int bt_decode_step(bt_model* m, int32_t batch, int32_t* next_ids_dev) {
  if (!m) return BT_ERR_ARG;
  const bt_config& c = m->cfg;
  if (!next_ids_dev) return fail(m, BT_ERR_ARG, "next_ids_dev is null");
  if (m->batch == 0) return fail(m, BT_ERR_STATE, "decode before prefill");
  if (batch != m->batch) return fail(m, BT_ERR_STATE, "batch differs from the prefill's");
  const Layout& L = m->L;
  const int r = m->r;
  const bool with_block = r == 0 && !m->have_context;
  if (with_block && m->n_blocks >= c.max_blocks) return fail(m, BT_ERR_CAPACITY, "block KV cache is full");
  hipStream_t s = m->stream;

  // A step kind (position in the block, with or without the block decoder) is a fixed launch
  // sequence: the count of cached blocks is read from device memory.  Its first occurrence runs
  // eagerly, the second is captured into a graph, later ones replay it.
  const int kind = with_block ? c.block_len : r;
  bool done = false;
  if (m->graphs_ok && c.use_graphs && !m->profile) {
    bt_model::StepGraph& g = m->graphs[kind];
    // A failed capture or instantiation is not an error of the step (it then runs eagerly, now and
    // from here on) but it is recorded: bt_stats.graph_fallback, and the reason in bt_last_error.
    auto give_up = [&](const char* what, hipError_t e) {
      m->graphs_ok = false;
      m->err = std::string("HIP graph ") + what + " failed (" + hipGetErrorString(e) + "): decode steps are launched eagerly";
      (void)hipGetLastError();
    };
    if (g.exec) {
      BT_HIP(m, hipGraphLaunch(g.exec, s));
      done = true;
    } else if (g.seen >= 1) {
      hipGraph_t graph = nullptr;
      hipError_t e = hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal);
      if (e == hipSuccess) {
        const int rc = enqueue_step(m, r, with_block, nullptr);
        e = hipStreamEndCapture(s, &graph);
        if (rc != BT_OK || e != hipSuccess || !graph) {
          if (graph) (void)hipGraphDestroy(graph);
          give_up("capture", e != hipSuccess ? e : hipErrorUnknown);
        } else {
          e = hipGraphInstantiate(&g.exec, graph, nullptr, nullptr, 0);
          (void)hipGraphDestroy(graph);
          if (e != hipSuccess) { g.exec = nullptr; give_up("instantiation", e); }
          else {
            m->graph_captures += 1;
            BT_HIP(m, hipGraphLaunch(g.exec, s));
            done = true;
          }
        }
      } else {
        give_up("capture", e);
      }
    }
    g.seen += 1;
  }
  if (done) m->graph_launches += 1;
  if (done) {
    BT_HIP(m, launch_gather_ids(m->at<int32_t>(L.cur), next_ids_dev, batch, c.block_len, r, s));
  } else {
    const int rc = enqueue_step(m, r, with_block, next_ids_dev);
    if (rc) return rc;
  }
  const int rows = r == 0 ? L.n_pref : 1, pos0 = r == 0 ? 0 : L.n_pref + r - 1;
  if (with_block) {
    m->st.block_passes += 1;
    m->st.block_kv_rows_read += m->n_blocks + 1;
    m->st.block_kv_bytes_read += (m->blocks_sum + batch) * c.n_block_layers * 2 * c.d_model * L.esz;
    m->n_blocks += 1;
    m->blocks_sum += batch;
  }
  if (r == 0) m->have_context = false;
  m->st.token_passes += 1;
  m->st.token_rows += rows;
  if (c.n_token_layers > 0 && pos0 + rows > m->st.local_kv_high_water) m->st.local_kv_high_water = pos0 + rows;
  m->r = (r + 1) % c.block_len;
  m->stepped = true;
  return BT_OK;
}

int bt_embed(bt_model* m, const int32_t* tokens_dev, int32_t n_rows, float* out_dev) {
  if (!m) return BT_ERR_ARG;
  if (!tokens_dev || !out_dev || n_rows < 0) return fail(m, BT_ERR_ARG, "bt_embed: null pointer or negative n_rows");
  BT_HIP(m, launch_embed_concat(m->cfg.dtype, m->w.E_emb, tokens_dev, out_dev, n_rows, 1, m->cfg.block_len,
                                m->cfg.d_model / m->cfg.block_len, m->cfg.block_len, m->cfg.block_len, nullptr,
                                m->cfg.pad_id, m->stream));
  return BT_OK;
}

int bt_score(bt_model* m, const int32_t* tokens_dev, int32_t batch, int32_t len, float* nll_dev) {
  if (!m) return BT_ERR_ARG;
  const bt_config& c = m->cfg;
  const Layout& L = m->L;
  if (!tokens_dev || !nll_dev) return fail(m, BT_ERR_ARG, "tokens_dev or nll_dev is null");
  if (c.score_rows < 1) return fail(m, BT_ERR_STATE, "the model was created with score_rows == 0");
  if (c.prefix_len < 1) return fail(m, BT_ERR_ARG, "scoring needs prefix_len >= 1");
  if (c.d_ff < c.d_model) return fail(m, BT_ERR_ARG, "scoring needs d_ff >= d_model");   // the context rows borrow the MLP buffer
  if (batch < 1 || batch > c.max_batch) return fail(m, BT_ERR_ARG, "batch out of range");
  if (len <= c.block_len) return fail(m, BT_ERR_ARG, "len must exceed block_len (two blocks or more after left padding)");
  const int N = (len + c.block_len - 1) / c.block_len, P = c.prefix_len, D = c.d_model, H = c.n_heads, dh = D / H;
  if (N > c.max_blocks) return fail(m, BT_ERR_CAPACITY, "more blocks than max_blocks");
  const int Lq = P + c.block_len - 1;
  const int per = L.m_rows / (N * Lq);          // sequences per chunk: all their token-decoder rows fit the workspace
  if (per < 1) return fail(m, BT_ERR_CAPACITY, "workspace rows < blocks * (prefix_len + block_len - 1)");
  hipStream_t s = m->stream;
  m->batch = 0;                                 // the block KV cache is overwritten: any generation state is gone
  m->have_context = false;
  m->stepped = false;
  drop_graphs(m);
  BT_HIP(m, hipMemsetAsync(nll_dev, 0, (size_t)batch * len * sizeof(float), s));
  const bool lo_planes = c.dtype == BT_BF16 && c.act_split >= 1;
  const size_t loD = lo_planes ? (size_t)L.m_rows * D : 0;
  float* x = m->at<float>(L.x);
  char* ctx_all = m->ws + L.hmid;               // free once the block stack's last GEMM has read it
  float* pref = m->at<float>(L.part_o);         // free after the stack's final LayerNorm
  char* h_all = m->ws + L.u1;                   // final hidden rows of the token decoder
  for (int b0 = 0; b0 < batch; b0 += per) {
    const int bc = batch - b0 < per ? batch - b0 : per;
    const int32_t* toks = tokens_dev + (size_t)b0 * len;
    // block decoder over all blocks; its final LayerNorm keeps every row: context j serves block j + 1
    BT_HIP(m, launch_embed_concat(c.dtype, m->w.E_emb, toks, x, bc, N, c.block_len, D / c.block_len, len, len, nullptr,
                                  c.pad_id, s));
    StackArgs ab{MODE_BLOCK_PREFILL, bc * N, bc, b0, N, 0};
    ab.fin_lo_off = loD;
    int rc = run_stack(m, m->blk.data(), c.n_block_layers, ab, m->w.blk_lnf_g, m->w.blk_lnf_b, ctx_all, 0, bc * N, 1, 0);
    if (rc) return rc;
    GemmProblem pp{ctx_all, m->w.W_prefix, (const float*)m->w.b_prefix, pref, bc * N, P * D, D, D, P * D, EPI_F32,
                   lo_planes ? ctx_all + loD * 2 : nullptr, 0, m->prefix_frag};
    GemmPlan pl{};
    BT_HIP(m, gemm_plan(c.dtype, &pp, 1, &pl));
    BT_HIP(m, launch_gemm(c.dtype, &pp, 1, pl, s));
    // token decoder over bc * (N - 1) independent local sequences of Lq rows
    BT_HIP(m, launch_score_assemble(c.dtype, pref, m->w.E_tok, toks, x, bc, N, len, D, P, c.block_len, s));
    const int n_loc = bc * (N - 1), rows = n_loc * Lq;
    StackArgs at{MODE_TOKEN, rows, n_loc, 0, Lq, 0};
    at.fin_lo_off = loD;
    at.loc_base = m->ws + L.score_kv;
    at.loc_half = (size_t)n_loc * H * L.l_cap * dh * L.esz;
    rc = run_stack(m, m->tok.data(), c.n_token_layers, at, m->w.tok_lnf_g, m->w.tok_lnf_b, h_all, 0, rows, 1, 0);
    if (rc) return rc;
    // LM head and log-softmax, score_rows rows at a time.  Where the tiled MFMA kernel serves the
    // head it leaves (max, sum of exponentials) per 64 columns and the target's logit instead of
    // the logits themselves; otherwise the logits go through memory and a kernel reduces each row.
    // The logits buffer holds, for the first form: stats | target logits | targets of the chunk.
    const int groups = (c.vocab + 63) / 64;
    float2* stats = m->at<float2>(L.score_logits);
    float* tgt_logit = reinterpret_cast<float*>(stats + (size_t)c.score_rows * groups);
    int32_t* targets = reinterpret_cast<int32_t*>(tgt_logit + c.score_rows);
    bool targets_made = false;
    for (int r0 = 0; r0 < rows; r0 += c.score_rows) {
      const int rc_rows = rows - r0 < c.score_rows ? rows - r0 : c.score_rows;
      GemmProblem ph{h_all + (size_t)r0 * D * L.esz, m->w.W_head, nullptr, m->ws + L.score_logits, rc_rows, c.vocab, D, D,
                     c.vocab, EPI_F32, lo_planes ? h_all + (loD + (size_t)r0 * D) * 2 : nullptr, 0, m->head_frag};
      GemmPlan ph_plan{};
      BT_HIP(m, gemm_plan(c.dtype, &ph, 1, &ph_plan));
      const bool fused = gemm_has_lse_epilogue(ph_plan) && (size_t)rows <= L.score_target_cap;
      if (fused) {
        if (!targets_made) {
          BT_HIP(m, launch_score_targets(toks, targets, rows, P, c.block_len, N, len, s));
          targets_made = true;
        }
        ph.epi = EPI_LSE;
        ph.out = stats;
        ph.lse_targets = targets + r0;
        ph.lse_target_out = tgt_logit;
      }
      int prc;
      if (m->profile && (prc = prof_begin(m, 2))) return prc;
      BT_HIP(m, launch_gemm(c.dtype, &ph, 1, ph_plan, s));
      if (m->profile) {
        if ((prc = prof_end(m))) return prc;
        m->st.gemm_tiled_launches += 1;
        m->st.gemm_tiled_flops += (int64_t)2 * rc_rows * c.vocab * D;
      }
      if (fused)
        BT_HIP(m, launch_score_combine(stats, groups, tgt_logit, rc_rows, r0, nll_dev + (size_t)b0 * len, P, c.block_len,
                                       N, len, s));
      else
        BT_HIP(m, launch_score_rows(m->at<float>(L.score_logits), rc_rows, c.vocab, r0, toks, nll_dev + (size_t)b0 * len,
                                    P, c.block_len, N, len, s));
    }
  }
  return BT_OK;
}

int bt_get_finished(bt_model* m, int32_t* flags_dev) {
  if (!m) return BT_ERR_ARG;
  if (!flags_dev) return fail(m, BT_ERR_ARG, "flags_dev is null");
  if (m->batch == 0) return fail(m, BT_ERR_STATE, "no prefill yet");
  BT_HIP(m, launch_gather_ids(m->at<int32_t>(m->L.fin), flags_dev, m->batch, 1, 0, m->stream));
  return BT_OK;
}

int bt_get_logits(bt_model* m, float* logits_dev) {
  if (!m) return BT_ERR_ARG;
  if (!logits_dev) return fail(m, BT_ERR_ARG, "logits_dev is null");
  if (!m->stepped || m->batch == 0) return fail(m, BT_ERR_STATE, "no decode step since the last prefill");
  if (!m->cfg.keep_logits) return fail(m, BT_ERR_STATE, "the model was created with keep_logits == 0");
  BT_HIP(m, hipMemcpyAsync(logits_dev, m->ws + m->L.logits, (size_t)m->batch * m->cfg.vocab * 4,
                           hipMemcpyDeviceToDevice, m->stream));
  return BT_OK;
}

int bt_force_last_ids(bt_model* m, const int32_t* ids_dev) {
  if (!m) return BT_ERR_ARG;
  if (!ids_dev) return fail(m, BT_ERR_ARG, "ids_dev is null");
  if (!m->stepped || m->batch == 0) return fail(m, BT_ERR_STATE, "no decode step since the last prefill");
  const int L_B = m->cfg.block_len;
  BT_HIP(m, launch_scatter_ids(ids_dev, m->at<int32_t>(m->L.cur), m->batch, L_B, (m->r + L_B - 1) % L_B, m->cfg.eos_id,
                               m->at<int32_t>(m->L.fin), m->stream));
  return BT_OK;
}

int bt_get_context(bt_model* m, void* ctx_dev) {
  if (!m) return BT_ERR_ARG;
  if (!ctx_dev) return fail(m, BT_ERR_ARG, "ctx_dev is null");
  if (m->batch == 0) return fail(m, BT_ERR_STATE, "no prefill yet");
  const size_t esz = m->cfg.prefix_len == 0 ? 4 : m->L.esz;
  BT_HIP(m, hipMemcpyAsync(ctx_dev, m->ws + m->L.ctx, (size_t)m->batch * m->cfg.d_model * esz, hipMemcpyDeviceToDevice, m->stream));
  return BT_OK;
}

int bt_set_context(bt_model* m, const void* ctx_dev) {
  if (!m) return BT_ERR_ARG;
  if (!ctx_dev) return fail(m, BT_ERR_ARG, "ctx_dev is null");
  if (m->batch == 0) return fail(m, BT_ERR_STATE, "no prefill yet");
  const size_t esz = m->cfg.prefix_len == 0 ? 4 : m->L.esz;
  BT_HIP(m, hipMemcpyAsync(m->ws + m->L.ctx, ctx_dev, (size_t)m->batch * m->cfg.d_model * esz, hipMemcpyDeviceToDevice, m->stream));
  if (m->cfg.prefix_len > 0 && m->cfg.dtype == BT_BF16 && m->cfg.act_split >= 1)   // remainder plane of an injected context is zero
    BT_HIP(m, hipMemsetAsync(m->ws + m->L.ctx + (size_t)m->cfg.max_batch * m->cfg.d_model * 2, 0,
                             (size_t)m->batch * m->cfg.d_model * 2, m->stream));
  return BT_OK;
}

int bt_set_profile(bt_model* m, int32_t on) {
  if (!m) return BT_ERR_ARG;
  m->profile = on != 0;
  return BT_OK;
}

int bt_probe_read(const void* src_dev, size_t bytes, void* hip_stream, float* out_dev) {
  if (!src_dev || !out_dev || bytes == 0 || bytes % BT_PROBE_READ_GRAIN) return BT_ERR_ARG;
  return launch_probe_read(src_dev, bytes, BT_PROBE_WORKGROUPS, out_dev, (hipStream_t)hip_stream) == hipSuccess ? BT_OK : BT_ERR_HIP;
}

int bt_probe_mfma(int32_t iters, int32_t random_operands, void* hip_stream, float* out_dev) {
  if (!out_dev || iters <= 0) return BT_ERR_ARG;
  return launch_probe_mfma(iters, random_operands, BT_PROBE_WORKGROUPS, out_dev, (hipStream_t)hip_stream) == hipSuccess ? BT_OK : BT_ERR_HIP;
}

int bt_reset_profile(bt_model* m) {
  if (!m) return BT_ERR_ARG;
  BT_HIP(m, hipStreamSynchronize(m->stream));
  m->ev_used = 0;
  m->st.attn_block_ms = 0.0;
  m->st.attn_block_launches = 0;
  m->st.attn_block_bytes = 0;
  m->st.gemm_decode_ms = 0.0;
  m->st.gemm_decode_launches = 0;
  m->st.gemm_decode_bytes = 0;
  m->st.gemm_tiled_ms = 0.0;
  m->st.gemm_tiled_launches = 0;
  m->st.gemm_tiled_flops = 0;
  return BT_OK;
}

int bt_get_stats(bt_model* m, bt_stats* out) {
  if (!m || !out) return BT_ERR_ARG;
  if (m->ev_used > 0) {
    BT_HIP(m, hipStreamSynchronize(m->stream));
    double ms[3] = {0.0, 0.0, 0.0};
    for (size_t i = 0; i + 1 < m->ev_used; i += 2) {
      float t = 0.f;
      BT_HIP(m, hipEventElapsedTime(&t, m->ev[i], m->ev[i + 1]));
      const int tag = m->ev_tag[i / 2];
      ms[tag >= 0 && tag <= 2 ? tag : 0] += t;
    }
    m->st.attn_block_ms = ms[0];
    m->st.gemm_decode_ms = ms[1];
    m->st.gemm_tiled_ms = ms[2];
  }
  m->st.n_blocks = m->n_blocks;
  m->st.r = m->r;
  m->st.batch = m->batch;
  m->st.graph_launches = m->graph_launches;
  m->st.graph_captures = m->graph_captures;
  m->st.graph_fallback = (m->cfg.use_graphs && !m->graphs_ok) ? 1 : 0;
  *out = m->st;
  return BT_OK;
}

const char* bt_last_error(const bt_model* m) { return m ? m->err.c_str() : g_create_err.c_str(); }

void bt_destroy(bt_model* m) {
  if (!m) return;
  if (m->static_dev >= 0) {
    // the next model on the static workspace may overwrite it at once: let this one's work drain first
    (void)hipStreamSynchronize(m->stream);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_owner[m->static_dev] == m) g_scratch_owner[m->static_dev] = nullptr;
  }
  for (hipEvent_t e : m->ev) (void)hipEventDestroy(e);
  for (auto& g : m->graphs) if (g.exec) (void)hipGraphExecDestroy(g.exec);
  delete m;
}

}  // extern "C"
