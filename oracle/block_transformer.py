"""CPU oracle for the Block Transformer generation step.  TEST INFRASTRUCTURE.

A plain, slow float64 numpy statement of what the model computes, written from
the paper's definitions (arXiv 2406.02657): embedder (Sec. 2.2, App. D.1
"Lookup"), block decoder (Sec. 2.3), token decoder with prefix tokens (Sec. 2.4,
App. D.2 "Prefix"), the inference procedure (Sec. 2.1, Fig. 1, App. C) and the
Pythia / GPT-NeoX layer type (Sec. 3.1, App. E.1).  Only tests, the smoke check
and the benchmark's cpu_baseline leg may import this package; the product path
never does, and nothing here imports the HIP path.

The method is exact (an architecture, not an approximation), so the oracle is
the definition written out.  Two ways to evaluate it are provided and tested
equal: "full" (no caches: recompute everything from the token history) and
"cached" (block-level KV cache plus a per-block local KV cache, the order the
GPU path follows).  Library primitives used as steps: numpy matmul, exp, sqrt,
and scipy's erf.

Readings taken where the paper is silent (each also listed in the design notes):
  * layer: pre-LayerNorm; parallel residual x + Attn(LN1 x) + MLP(LN2 x) by
    default (Pythia), sequential wiring selectable;
  * rotary position rotation on the first `rot` dims of every head, pairing
    dim t with t + rot/2, angle pos * 10000^(-2t/rot); block decoder position =
    block index, token decoder position = index inside the local sequence;
  * the output at the last prefix position predicts the first token of a block;
    the last token of a block is never fed to the token decoder;
  * prefix projection is one affine map D -> P*D; both decoders end in a final
    LayerNorm; exact (erf) GELU; biased variance, eps inside the square root;
    LM head has no bias; greedy argmax, lowest index on ties;
  * prefix_len == 0 (only with block_len == 1): the context embedding itself is
    the token decoder's single input row;
  * a prompt whose length is not a multiple of L_B gets the fewest pad tokens
    (0 .. L_B-1 of cfg.pad_id) in FRONT of its first block; the pads are
    embedded like any token (App. "Random length padding", footnote of the
    zero-shot table in Sec. 3);
  * the "Summation" token decoder of App. D.2 (cfg.token_mix == "sum"): the context embedding is
    projected to L_B vectors of dimension D and vector k is added to the token decoder's input at
    local position k.  The paper does not say what token embedding stands at position 0, the
    position that predicts the block's first token (no token of the block is known yet, and the
    token decoder sees nothing outside the block): here none does, input 0 is vector 0 alone, and
    input k >= 1 is E_tok[token k-1 of the block] + vector k; the output at position k predicts
    token k.  prefix_len must be 1 (position bookkeeping is that of one prefix row);
  * stopping is not part of the paper (it generates a fixed number of tokens):
    with cfg.eos_id >= 0 a sequence that has emitted eos_id emits eos_id at
    every later step; the batch stays static and the other sequences are
    unaffected.
All arithmetic is float64 on the stored weight values (bf16 bit patterns are
widened exactly); nothing else is rounded.

Parity pins (tests/test_oracle_*.py): cached == full; locality and causality;
reduction to an independently written vanilla transformer at L_B = 1;
brute-force attention; closed forms (running mean, constant logits, one-hot
head); rotary relative-position invariance; operation counts the paper states;
the bf16 storage path (hand-computed values of bit patterns, round-to-nearest-
even cases, cached == full on bf16 weights, bit-equal to float32 weights that
hold the widened values); the summation variant (cached == full, reduction to
the one-prefix model, causal effect of each summand, inputs written out).
The numeric value of a logit is otherwise unpinned: the paper prints no worked
example.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf


# ----------------------------------------------------------------------------
# parameters
# ----------------------------------------------------------------------------
class Params:
    """Read-only view of a weight dict that hands out float64 arrays.

    uint16 arrays are bf16 bit patterns and are widened exactly.  With
    keep=True the widened copies are kept (fast repeated decode steps); with
    keep=False each access converts afresh (small memory at large configs).
    """

    def __init__(self, weights, keep=True):
        self._w = weights
        self._keep = keep
        self._c = {}

    def __contains__(self, name):
        return name in self._w

    def __call__(self, name):
        if name in self._c:
            return self._c[name]
        a = self._w[name]
        if a.dtype == np.uint16:
            a = (a.astype(np.uint32) << np.uint32(16)).view(np.float32)
        a = a.astype(np.float64)
        if self._keep:
            self._c[name] = a
        return a


# ----------------------------------------------------------------------------
# elementary pieces of the layer (Pythia / GPT-NeoX type, Sec. 3.1)
# ----------------------------------------------------------------------------
def layer_norm(x, gamma, beta, eps):
    mean = x.mean(axis=-1, keepdims=True)
    var = ((x - mean) ** 2).mean(axis=-1, keepdims=True)      # biased
    return (x - mean) / np.sqrt(var + eps) * gamma + beta


def gelu(u):
    return 0.5 * u * (1.0 + erf(u / np.sqrt(2.0)))


def rotary(x, pos, rot):
    """Rotate the first `rot` dims of every head.  x: [B, n, H, d_h]; pos: [n]."""
    if rot == 0:
        return x
    half = rot // 2
    t = np.arange(half, dtype=np.float64)
    inv_freq = 10000.0 ** (-2.0 * t / rot)                     # [half]
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]   # [n, half]
    cos = np.cos(ang)[None, :, None, :]
    sin = np.sin(ang)[None, :, None, :]
    lo, hi = x[..., :half], x[..., half:rot]
    out = x.copy()
    out[..., :half] = lo * cos - hi * sin
    out[..., half:rot] = hi * cos + lo * sin
    return out


def attention(q, K, V, n_past):
    """Causal softmax attention.

    q: [B, n, H, d_h] queries for positions n_past .. n_past+n-1;
    K, V: [B, n_past+n, H, d_h] keys/values for positions 0 .. n_past+n-1.
    Query i sees keys 0 .. n_past+i.  Returns [B, n, H, d_h].
    """
    d_h = q.shape[-1]
    n, n_k = q.shape[1], K.shape[1]
    s = np.matmul(q.transpose(0, 2, 1, 3), K.transpose(0, 2, 3, 1)) / np.sqrt(d_h)   # [B,H,n,n_k]
    i = np.arange(n)[:, None]
    j = np.arange(n_k)[None, :]
    s = np.where(j <= n_past + i, s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    o = np.matmul(p, V.transpose(0, 2, 1, 3))                                        # [B,H,n,d_h]
    return o.transpose(0, 2, 1, 3)


class LayerCache:
    """K and V of one layer for positions 0 .. n-1 of every sequence in the batch."""

    def __init__(self, batch, capacity, n_heads, d_head):
        self.K = np.zeros((batch, capacity, n_heads, d_head))
        self.V = np.zeros((batch, capacity, n_heads, d_head))
        self.n = 0

    def append(self, k, v):
        m = k.shape[1]
        self.K[:, self.n:self.n + m] = k
        self.V[:, self.n:self.n + m] = v
        self.n += m

    def clear(self):
        self.n = 0


def transformer_layer(P, prefix, x, pos0, cfg, cache=None):
    """One decoder layer on rows x [B, n, D] sitting at positions pos0 .. pos0+n-1.

    Without a cache, pos0 must be 0 and the rows are the whole sequence.  With a
    cache holding positions 0 .. pos0-1, the new K,V are appended to it.
    """
    B, n, D = x.shape
    H, d_h = cfg.n_heads, cfg.d_head
    w = lambda nm: P(prefix + nm)
    pos = np.arange(pos0, pos0 + n)

    def attn_branch(inp):
        u = layer_norm(inp, w("ln1_g"), w("ln1_b"), cfg.ln_eps)
        qkv = u @ w("W_qkv").T + w("b_qkv")
        q = qkv[..., 0 * D:1 * D].reshape(B, n, H, d_h)
        k = qkv[..., 1 * D:2 * D].reshape(B, n, H, d_h)
        v = qkv[..., 2 * D:3 * D].reshape(B, n, H, d_h)
        q = rotary(q, pos, cfg.rot)
        k = rotary(k, pos, cfg.rot)
        if cache is None:
            assert pos0 == 0
            K, V = k, v
        else:
            assert cache.n == pos0
            cache.append(k, v)
            K, V = cache.K[:, :cache.n], cache.V[:, :cache.n]
        o = attention(q, K, V, pos0).reshape(B, n, D)
        return o @ w("W_o").T + w("b_o")

    def mlp_branch(inp):
        u = layer_norm(inp, w("ln2_g"), w("ln2_b"), cfg.ln_eps)
        return gelu(u @ w("W_up").T + w("b_up")) @ w("W_down").T + w("b_down")

    if cfg.parallel_residual:
        return x + attn_branch(x) + mlp_branch(x)
    y = x + attn_branch(x)
    return y + mlp_branch(y)


# ----------------------------------------------------------------------------
# the three components (Sec. 2.2 - 2.4)
# ----------------------------------------------------------------------------
def embedder(P, cfg, tokens):
    """tokens [B, n*L_B] -> block embeddings [B, n, D]: lookup in E_emb and concatenate."""
    B, T = tokens.shape
    L_B = cfg.block_len
    assert T % L_B == 0
    rows = P("E_emb")[tokens]                       # [B, T, D_emb]
    return rows.reshape(B, T // L_B, L_B * cfg.d_emb)


def block_decoder(P, cfg, e, pos0=0, caches=None):
    """Block embeddings e [B, n, D] at block positions pos0.. -> context embeddings [B, n, D].

    Output j is the context embedding for block pos0+j+1 (it has seen blocks
    0 .. pos0+j).  Ends in the block decoder's final LayerNorm.
    """
    h = e
    for l in range(cfg.n_block_layers):
        h = transformer_layer(P, f"blk.{l}.", h, pos0, cfg, None if caches is None else caches[l])
    return layer_norm(h, P("blk_lnf_g"), P("blk_lnf_b"), cfg.ln_eps)


def prefix_tokens(P, cfg, c):
    """Context embeddings c [B, D] -> token-decoder prefix rows [B, max(P,1), D]."""
    B, D = c.shape
    if cfg.prefix_len == 0:
        assert cfg.block_len == 1
        return c.reshape(B, 1, D)
    return (c @ P("W_prefix").T + P("b_prefix")).reshape(B, cfg.prefix_len, D)


def summands(P, cfg, c):
    """Summation variant (App. D.2): context embeddings c [B, D] -> [B, L_B, D], one vector per
    local position of the token decoder."""
    B, D = c.shape
    return (c @ P("W_prefix").T + P("b_prefix")).reshape(B, cfg.block_len, D)


def local_inputs(P, cfg, c, block_tokens):
    """Input rows of the token decoder for one block: context c [B, D] and the block's first r tokens
    [B, r] -> [B, n_prefix_rows + r, D].

    Prefix variant: the prefix rows, then E_tok of the tokens.  Summation variant: position 0 holds
    summand 0 alone, position k >= 1 holds E_tok[token k-1] + summand k.
    """
    B, r = block_tokens.shape
    if getattr(cfg, "token_mix", "prefix") == "sum":
        assert cfg.prefix_len == 1
        u = summands(P, cfg, c)
        s = u[:, :r + 1].copy()
        if r > 0:
            s[:, 1:] += P("E_tok")[block_tokens]
        return s
    s = prefix_tokens(P, cfg, c)
    if r > 0:
        s = np.concatenate([s, P("E_tok")[block_tokens]], axis=1)
    return s


def token_decoder(P, cfg, s, pos0=0, caches=None):
    """Local sequence rows s [B, n, D] at local positions pos0.. -> hidden [B, n, D] after final LN."""
    g = s
    for l in range(cfg.n_token_layers):
        g = transformer_layer(P, f"tok.{l}.", g, pos0, cfg, None if caches is None else caches[l])
    return layer_norm(g, P("tok_lnf_g"), P("tok_lnf_b"), cfg.ln_eps)


def lm_head(P, hidden):
    return hidden @ P("W_head").T


def greedy(logits):
    """argmax over the last axis, lowest index on ties."""
    return np.argmax(logits, axis=-1).astype(np.int32)


def left_pad(cfg, prompts):
    """Fill the first block of prompts [B, T], T >= 1, from the left (App. "Random length padding").

    Returns [B, ceil(T/L_B)*L_B]: (-T mod L_B) copies of cfg.pad_id, then the prompt.  The
    pads are ordinary tokens from here on: the embedder looks them up and concatenates them
    into the first block's embedding.  A prompt of one token is the paper's setting without
    an input sequence (App. on batch sizes and context lengths): L_B - 1 pads and that token.
    """
    prompts = np.asarray(prompts, dtype=np.int64)
    B, T = prompts.shape
    assert T >= 1
    k = (-T) % cfg.block_len
    return np.concatenate([np.full((B, k), cfg.pad_id, dtype=np.int64), prompts], axis=1)


# ----------------------------------------------------------------------------
# mode "full": the plain definition, no caches
# ----------------------------------------------------------------------------
def context_embeddings(P, cfg, tokens):
    """tokens [B, n*L_B] (complete blocks 0..n-1) -> [B, n, D]; entry j is the context for block j+1."""
    return block_decoder(P, cfg, embedder(P, cfg, tokens))


def block_logits(P, cfg, c, block_tokens):
    """Logits of one block given its context embedding.

    c [B, D]; block_tokens [B, r] = the first r tokens of the block (0 <= r <= L_B-1).
    Returns [B, r+1, V]: entry k is the distribution of the block's token k
    (entry 0 comes from the last prefix position).
    """
    B, r = block_tokens.shape
    assert r <= max(cfg.block_len - 1, 0)
    s = local_inputs(P, cfg, c, block_tokens)
    g = token_decoder(P, cfg, s)
    return lm_head(P, g[:, cfg.n_prefix_rows - 1:])


def next_token_logits_full(P, cfg, tokens):
    """Definition of one generation step: history tokens [B, T], T >= L_B -> logits [B, V] for x_T."""
    B, T = tokens.shape
    L_B = cfg.block_len
    i, r = T // L_B, T % L_B
    assert i >= 1
    c = context_embeddings(P, cfg, tokens[:, :i * L_B])[:, -1]
    return block_logits(P, cfg, c, tokens[:, i * L_B:])[:, r]


def teacher_forced_logits(P, cfg, tokens, blocks):
    """Logits for every token of the chosen blocks, given the full history.

    tokens [B, T] with T a multiple of L_B; blocks: iterable of block indices
    i >= 1.  Returns {i: [B, L_B, V]} where entry [:, k] is the distribution of
    token i*L_B + k given tokens 0 .. i*L_B + k - 1.  Same definition as
    next_token_logits_full, evaluated for many positions from one block-decoder
    pass (valid because the block decoder is causal).
    """
    L_B = cfg.block_len
    ctx = context_embeddings(P, cfg, tokens[:, :(max(blocks)) * L_B])
    out = {}
    for i in blocks:
        assert i >= 1
        out[i] = block_logits(P, cfg, ctx[:, i - 1], tokens[:, i * L_B:(i + 1) * L_B - 1])
    return out


def score_nll(P, cfg, tokens):
    """Teacher-forced scoring (the training-time forward of Sec. 2.1 / Fig. 1: both decoders over all
    blocks at once).  tokens [B, T], any T that spans two blocks or more once its first block has been
    completed from the left (left_pad).

    Returns [B, T] float64: entry t is -log p(x_t | x_<t), the softmax of the logits that
    next_token_logits_full defines for that position; the tokens of the first block have no context
    embedding and are not scored (zeros).
    """
    tokens = np.asarray(tokens, dtype=np.int64)
    B, T = tokens.shape
    L_B = cfg.block_len
    padded = left_pad(cfg, tokens)
    pad = padded.shape[1] - T
    n = padded.shape[1] // L_B
    assert n >= 2
    lg = teacher_forced_logits(P, cfg, padded, range(1, n))
    out = np.zeros((B, padded.shape[1]))
    for i in range(1, n):
        z = lg[i]                                               # [B, L_B, V]
        zmax = z.max(axis=-1, keepdims=True)
        lse = zmax[..., 0] + np.log(np.exp(z - zmax).sum(axis=-1))
        tgt = padded[:, i * L_B:(i + 1) * L_B]
        out[:, i * L_B:(i + 1) * L_B] = lse - np.take_along_axis(z, tgt[..., None], axis=-1)[..., 0]
    return out[:, pad:]


def generate_full(P, cfg, prompts, n_new):
    """Greedy generation by full recomputation.  Returns (ids [B, n_new], logits [B, n_new, V])."""
    hist = left_pad(cfg, prompts)
    ids, lgs = [], []
    for _ in range(n_new):
        lg = next_token_logits_full(P, cfg, hist)
        nxt = greedy(lg)
        ids.append(nxt)
        lgs.append(lg)
        hist = np.concatenate([hist, nxt[:, None].astype(np.int64)], axis=1)
    return np.stack(ids, axis=1), np.stack(lgs, axis=1)


# ----------------------------------------------------------------------------
# mode "cached": prefill + one token per step (Sec. 2.1, Fig. 1, App. C)
# ----------------------------------------------------------------------------
class CachedGenerator:
    """Incremental generation with a block-level KV cache and a local KV cache.

    prefill(prompts) runs the block decoder over all prompt blocks (the token
    decoder is not run on prompt blocks) and keeps the last context embedding.
    step() emits one token per sequence; the block decoder runs once per L_B
    steps, lazily at the start of the step that opens a new block.
    """

    def __init__(self, P, cfg, batch, max_blocks):
        self.P, self.cfg, self.B = P, cfg, batch
        H, d_h = cfg.n_heads, cfg.d_head
        self.blk = [LayerCache(batch, max_blocks, H, d_h) for _ in range(cfg.n_block_layers)]
        self.loc = [LayerCache(batch, cfg.n_prefix_rows + cfg.block_len, H, d_h)
                    for _ in range(cfg.n_token_layers)]
        self.cur = np.zeros((batch, cfg.block_len), dtype=np.int64)   # tokens of the open block
        self.r = 0                      # tokens already generated in the open block
        self.n_blocks = 0               # blocks pushed through the block decoder so far
        self.have_context = False
        self.c = None
        # counters for the statements the paper makes about the procedure
        self.block_passes = 0           # block-decoder invocations (prefill counts once per block)
        self.token_passes = 0
        self.token_rows = 0             # rows pushed through the token decoder
        self.block_kv_rows_read = 0     # cached block entries attended, summed over decode steps
        self.local_kv_high_water = 0
        self.finished = np.zeros(batch, dtype=bool)   # has emitted cfg.eos_id (only when eos_id >= 0)

    def prefill(self, prompts):
        cfg = self.cfg
        prompts = left_pad(cfg, prompts)
        B, T = prompts.shape
        assert B == self.B and T >= cfg.block_len and T % cfg.block_len == 0
        for c in self.blk + self.loc:
            c.clear()
        ctx = block_decoder(self.P, cfg, embedder(self.P, cfg, prompts), 0, self.blk)
        self.block_passes = self.n_blocks = T // cfg.block_len
        self.c = ctx[:, -1]
        self.have_context = True
        self.r = 0
        self.token_passes = self.token_rows = self.block_kv_rows_read = 0
        self.local_kv_high_water = 0
        self.finished[:] = False

    def step(self, forced_ids=None):
        """One decode step.  Returns (logits [B, V], ids [B]).

        forced_ids, when given, replaces the greedy choice as the token that
        enters the history (teacher forcing); the returned ids are still the
        greedy ones.
        """
        P, cfg = self.P, self.cfg
        if self.r == 0:
            if not self.have_context:
                n_before = self.n_blocks
                e = embedder(P, cfg, self.cur)
                self.c = block_decoder(P, cfg, e, n_before, self.blk)[:, -1]
                self.block_passes += 1
                self.n_blocks += 1
                self.block_kv_rows_read += n_before + 1
            for c in self.loc:
                c.clear()
            s = local_inputs(P, cfg, self.c, self.cur[:, :0])
            self.have_context = False
        elif getattr(cfg, "token_mix", "prefix") == "sum":
            s = (P("E_tok")[self.cur[:, self.r - 1]] + summands(P, cfg, self.c)[:, self.r])[:, None, :]
        else:
            s = P("E_tok")[self.cur[:, self.r - 1]][:, None, :]
        g = token_decoder(P, cfg, s, self.loc[0].n if self.loc else 0, self.loc)
        self.token_passes += 1
        self.token_rows += s.shape[1]
        if self.loc:
            self.local_kv_high_water = max(self.local_kv_high_water, self.loc[0].n)
        logits = lm_head(P, g[:, -1])
        ids = greedy(logits)
        eos = getattr(cfg, "eos_id", -1)
        if eos >= 0:
            ids = np.where(self.finished, eos, ids).astype(np.int32)
            self.finished |= ids == eos
        fed = ids if forced_ids is None else np.asarray(forced_ids)
        self.cur[:, self.r] = fed
        self.r = (self.r + 1) % cfg.block_len
        return logits, ids


def generate_cached(P, cfg, prompts, n_new, forced=None):
    """Greedy (or teacher-forced on `forced` [B, n_new]) generation in cached mode."""
    prompts = np.asarray(prompts)
    B, T = prompts.shape
    gen = CachedGenerator(P, cfg, B, (T + n_new) // cfg.block_len + 2)
    gen.prefill(prompts)
    ids, lgs = [], []
    for t in range(n_new):
        lg, nxt = gen.step(None if forced is None else forced[:, t])
        ids.append(nxt)
        lgs.append(lg)
    return np.stack(ids, axis=1), np.stack(lgs, axis=1), gen


def generate_ragged(P, cfg, prompts, n_new, forced=None):
    """Prompts of different lengths in one batch: a list of 1-D id arrays, each of length >= 1.

    Sequences never interact (every attention and every table lookup is per sequence), so the
    batch is defined as each sequence generated alone, left-padded on its own (left_pad).
    forced: optional [B, n_new] ids fed back in place of the greedy choice.
    Returns (ids [B, n_new], logits [B, n_new, V]).
    """
    ids, lgs = [], []
    for b, p in enumerate(prompts):
        i, l, _ = generate_cached(P, cfg, np.asarray(p)[None, :], n_new,
                                  None if forced is None else np.asarray(forced)[b:b + 1])
        ids.append(i[0])
        lgs.append(l[0])
    return np.stack(ids), np.stack(lgs)
