"""ctypes binding of libbt.so: argument marshalling only.

PyTorch is used for device memory (weights, workspace, token and output
buffers) and for the current HIP stream; every step of the computation runs in
the library's kernels.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  first: libbt.so must bind to the HIP runtime torch brings, not load a second copy

HERE = os.path.dirname(os.path.abspath(__file__))
lib_path = os.path.join(HERE, "libbt.so")
if not os.path.exists(lib_path):
    raise ImportError(
        f"{lib_path} is missing: build it first (python -m paper_2406_02657_amd.build, "
        "or __graft_entry__.build()).  There is no fallback path.")
lib = C.CDLL(lib_path)

BT_F32, BT_BF16 = 0, 1
BT_MIX_PREFIX, BT_MIX_SUM = 0, 1
BT_OK, BT_ERR_ARG, BT_ERR_STATE, BT_ERR_CAPACITY, BT_ERR_HIP = 0, -1, -2, -3, -4


class bt_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "struct_size", "vocab", "block_len", "d_model", "n_heads", "d_ff", "n_block_layers", "n_token_layers",
        "prefix_len", "dtype", "max_batch", "max_blocks", "rotary_dims", "parallel_residual",
        "prefill_rows", "act_split", "use_graphs", "pad_id", "score_rows", "eos_id", "keep_logits",
        "token_mix")] + [("ln_eps", C.c_float)]


_LAYER_FIELDS = ("ln1_g", "ln1_b", "W_qkv", "b_qkv", "W_o", "b_o", "ln2_g", "ln2_b", "W_up", "b_up", "W_down", "b_down")


class bt_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _LAYER_FIELDS]


class bt_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in (
        "E_emb", "E_tok", "W_prefix", "b_prefix", "W_head", "blk_lnf_g", "blk_lnf_b", "tok_lnf_g", "tok_lnf_b")] + [
        ("block_layers", C.POINTER(bt_layer_weights)), ("token_layers", C.POINTER(bt_layer_weights))]


class bt_stats(C.Structure):
    _fields_ = [("block_passes", C.c_int64), ("token_passes", C.c_int64), ("token_rows", C.c_int64),
                ("block_kv_rows_read", C.c_int64), ("block_kv_bytes_read", C.c_int64),
                ("n_blocks", C.c_int32), ("r", C.c_int32), ("batch", C.c_int32),
                ("local_kv_high_water", C.c_int32), ("attn_block_ms", C.c_double),
                ("attn_block_launches", C.c_int64), ("attn_block_bytes", C.c_int64),
                ("gemm_decode_ms", C.c_double), ("gemm_decode_launches", C.c_int64),
                ("gemm_decode_bytes", C.c_int64), ("gemm_tiled_ms", C.c_double),
                ("gemm_tiled_launches", C.c_int64), ("gemm_tiled_flops", C.c_int64),
                ("graph_launches", C.c_int64), ("graph_captures", C.c_int32), ("graph_fallback", C.c_int32)]


_P = C.c_void_p
lib.bt_workspace_bytes.argtypes = [C.POINTER(bt_config), C.POINTER(C.c_size_t)]
lib.bt_create.argtypes = [C.POINTER(bt_config), C.POINTER(bt_weights), _P, C.c_size_t, _P, C.POINTER(_P)]
lib.bt_create_static.argtypes = [C.POINTER(bt_config), C.POINTER(bt_weights), _P, C.POINTER(_P)]
lib.bt_prefill.argtypes = [_P, _P, C.c_int32, C.c_int32]
lib.bt_prefill_ragged.argtypes = [_P, _P, C.POINTER(C.c_int32), C.c_int32, C.c_int32]
lib.bt_decode_step.argtypes = [_P, C.c_int32, _P]
lib.bt_get_logits.argtypes = [_P, _P]
lib.bt_get_finished.argtypes = [_P, _P]
lib.bt_score.argtypes = [_P, _P, C.c_int32, C.c_int32, _P]
lib.bt_force_last_ids.argtypes = [_P, _P]
lib.bt_get_context.argtypes = [_P, _P]
lib.bt_set_context.argtypes = [_P, _P]
lib.bt_set_profile.argtypes = [_P, C.c_int32]
lib.bt_reset_profile.argtypes = [_P]
lib.bt_get_stats.argtypes = [_P, C.POINTER(bt_stats)]
lib.bt_last_error.argtypes = [_P]
lib.bt_last_error.restype = C.c_char_p
lib.bt_destroy.argtypes = [_P]
lib.bt_destroy.restype = None
lib.bt_embed.argtypes = [_P, _P, C.c_int32, _P]
lib.bt_probe_read.argtypes = [_P, C.c_size_t, _P, _P]
lib.bt_probe_mfma.argtypes = [C.c_int32, C.c_int32, _P, _P]
PROBE_WORKGROUPS = 2048
PROBE_READ_GRAIN = PROBE_WORKGROUPS * 256 * 16
for _f in ("bt_workspace_bytes", "bt_create", "bt_create_static", "bt_prefill", "bt_prefill_ragged", "bt_decode_step", "bt_get_logits",
           "bt_get_finished", "bt_score", "bt_force_last_ids",
           "bt_get_context", "bt_set_context", "bt_set_profile", "bt_reset_profile", "bt_get_stats", "bt_embed",
           "bt_probe_read", "bt_probe_mfma"):
    getattr(lib, _f).restype = C.c_int


class BTError(RuntimeError):
    def __init__(self, code, msg=""):
        super().__init__(f"bt status {code}: {msg}")
        self.code = code


DEFAULT_ACT_SPLIT = 2


def make_config(cfg, max_batch=None, max_blocks=None, prefill_rows=0, act_split=None, use_graphs=1,
                score_rows=0, keep_logits=1) -> bt_config:
    """cfg: any object with the fields of synth.BTConfig."""
    return bt_config(
        struct_size=C.sizeof(bt_config), vocab=cfg.vocab, block_len=cfg.block_len, d_model=cfg.d_model, n_heads=cfg.n_heads, d_ff=cfg.d_ff,
        n_block_layers=cfg.n_block_layers, n_token_layers=cfg.n_token_layers, prefix_len=cfg.prefix_len,
        dtype=BT_BF16 if cfg.dtype == "bf16" else BT_F32,
        max_batch=cfg.batch if max_batch is None else max_batch,
        max_blocks=cfg.max_blocks if max_blocks is None else max_blocks,
        rotary_dims=cfg.rot, parallel_residual=cfg.parallel_residual, prefill_rows=prefill_rows,
        act_split=DEFAULT_ACT_SPLIT if act_split is None else act_split,
        use_graphs=int(use_graphs),
        pad_id=getattr(cfg, "pad_id", 0), score_rows=score_rows, eos_id=getattr(cfg, "eos_id", -1),
        keep_logits=int(keep_logits),
        token_mix=BT_MIX_SUM if getattr(cfg, "token_mix", "prefix") == "sum" else BT_MIX_PREFIX, ln_eps=cfg.ln_eps)


class _Ordered:
    """Orders one library call (enqueued on `stream`) against torch's current stream."""

    def __init__(self, torch, device, stream):
        self.cur = torch.cuda.current_stream(device)
        self.stream = stream

    def __enter__(self):
        if self.cur != self.stream:
            self.stream.wait_stream(self.cur)

    def __exit__(self, *exc):
        if self.cur != self.stream:
            self.cur.wait_stream(self.stream)
        return False


class Model:
    """Owns the device copies of the weights and the workspace; forwards to the C ABI."""

    def __init__(self, cfg, weights, max_batch=None, max_blocks=None, prefill_rows=0, act_split=None,
                 use_graphs=1, score_rows=0, keep_logits=1, device="cuda:0", stream=None, static_workspace=False):
        import torch
        self.torch = torch
        self.device = torch.device(device)
        self.cfg = cfg
        self.c = make_config(cfg, max_batch, max_blocks, prefill_rows, act_split, use_graphs, score_rows, keep_logits)
        # The library enqueues everything on one HIP stream.  HIP graphs cannot be captured on the
        # default stream, so the model brings a stream of its own (default priority).  Callers
        # that make it current (`with model.on_stream():`) pay nothing; from any other stream
        # every call is bracketed by the two stream waits that keep the order.
        self.stream = torch.cuda.Stream(self.device) if stream is None else stream
        self._keep = {}
        for name, arr in weights.items():
            a = np.ascontiguousarray(arr)
            t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(self.device)
            self._keep[name] = t
        ptr = lambda n: self._keep[n].data_ptr() if n in self._keep else None

        def layers(stack, n):
            arr = (bt_layer_weights * max(n, 1))()
            for i in range(n):
                for f in _LAYER_FIELDS:
                    setattr(arr[i], f, ptr(f"{stack}.{i}.{f}"))
            return arr

        self._blk = layers("blk", cfg.n_block_layers)
        self._tok = layers("tok", cfg.n_token_layers)
        self.w = bt_weights(E_emb=ptr("E_emb"), E_tok=ptr("E_tok"), W_prefix=ptr("W_prefix"), b_prefix=ptr("b_prefix"),
                            W_head=ptr("W_head"), blk_lnf_g=ptr("blk_lnf_g"), blk_lnf_b=ptr("blk_lnf_b"),
                            tok_lnf_g=ptr("tok_lnf_g"), tok_lnf_b=ptr("tok_lnf_b"),
                            block_layers=self._blk, token_layers=self._tok)
        nbytes = C.c_size_t(0)
        rc = lib.bt_workspace_bytes(C.byref(self.c), C.byref(nbytes))
        if rc:
            raise BTError(rc, "bt_workspace_bytes")
        self.workspace_bytes = nbytes.value
        self.h = _P()
        if static_workspace:
            # bt_create_static: the workspace is the library's static device array; nothing is allocated here
            self.workspace = None
            with self.torch.cuda.device(self.device), self._ordered():
                rc = lib.bt_create_static(C.byref(self.c), C.byref(self.w), self.stream.cuda_stream, C.byref(self.h))
        else:
            self.workspace = torch.empty(nbytes.value + 256, dtype=torch.uint8, device=self.device)
            base = (self.workspace.data_ptr() + 255) // 256 * 256
            with self._ordered():
                rc = lib.bt_create(C.byref(self.c), C.byref(self.w), base, nbytes.value, self.stream.cuda_stream,
                                   C.byref(self.h))
        if rc:
            raise BTError(rc, (lib.bt_last_error(None) or b"").decode())
        self.batch = 0

    def on_stream(self):
        """Context manager that makes the model's stream torch's current stream."""
        return self.torch.cuda.stream(self.stream)

    def _ordered(self):
        return _Ordered(self.torch, self.device, self.stream)

    def _chk(self, rc):
        if rc:
            raise BTError(rc, (lib.bt_last_error(self.h) or b"").decode())

    def bt_prefill(self, tokens):
        """tokens: int32 cuda tensor [batch, prompt_len]."""
        assert tokens.dtype == self.torch.int32 and tokens.is_cuda and tokens.is_contiguous()
        with self._ordered():
            self._chk(lib.bt_prefill(self.h, tokens.data_ptr(), tokens.shape[0], tokens.shape[1]))
        self._after_prefill(tokens.shape[0])

    def bt_prefill_ragged(self, tokens, lens):
        """tokens: int32 cuda tensor [batch, max_len]; lens: host sequence of batch prompt lengths."""
        assert tokens.dtype == self.torch.int32 and tokens.is_cuda and tokens.is_contiguous()
        assert len(lens) == tokens.shape[0]
        arr = (C.c_int32 * len(lens))(*[int(v) for v in lens])
        with self._ordered():
            self._chk(lib.bt_prefill_ragged(self.h, tokens.data_ptr(), arr, tokens.shape[0], tokens.shape[1]))
        self._after_prefill(tokens.shape[0])

    def _after_prefill(self, batch):
        self.batch = batch
        self._ids = self.torch.empty(self.batch, dtype=self.torch.int32, device=self.device)

    def bt_decode_step(self, out=None):
        ids = self._ids if out is None else out
        with self._ordered():
            self._chk(lib.bt_decode_step(self.h, self.batch, ids.data_ptr()))
        return ids

    def bt_get_logits(self):
        lg = self.torch.empty(self.batch, self.cfg.vocab, dtype=self.torch.float32, device=self.device)
        with self._ordered():
            self._chk(lib.bt_get_logits(self.h, lg.data_ptr()))
        return lg

    def bt_score(self, tokens):
        """tokens: int32 cuda tensor [batch, len]; returns float32 [batch, len] negative log-likelihoods."""
        assert tokens.dtype == self.torch.int32 and tokens.is_cuda and tokens.is_contiguous()
        nll = self.torch.empty(tokens.shape, dtype=self.torch.float32, device=self.device)
        with self._ordered():
            self._chk(lib.bt_score(self.h, tokens.data_ptr(), tokens.shape[0], tokens.shape[1], nll.data_ptr()))
        return nll

    def bt_get_finished(self):
        fl = self.torch.empty(self.batch, dtype=self.torch.int32, device=self.device)
        with self._ordered():
            self._chk(lib.bt_get_finished(self.h, fl.data_ptr()))
        return fl

    def bt_force_last_ids(self, ids):
        assert ids.dtype == self.torch.int32 and ids.is_cuda
        with self._ordered():
            self._chk(lib.bt_force_last_ids(self.h, ids.data_ptr()))

    def _ctx_dtype(self):
        if self.cfg.prefix_len == 0 or self.cfg.dtype != "bf16":
            return self.torch.float32
        return self.torch.bfloat16

    def bt_get_context(self):
        c = self.torch.empty(self.batch, self.cfg.d_model, dtype=self._ctx_dtype(), device=self.device)
        with self._ordered():
            self._chk(lib.bt_get_context(self.h, c.data_ptr()))
        return c

    def bt_set_context(self, c):
        assert c.dtype == self._ctx_dtype() and c.is_cuda and c.is_contiguous()
        with self._ordered():
            self._chk(lib.bt_set_context(self.h, c.data_ptr()))

    def bt_embed(self, tokens):
        """Embedder alone: int32 cuda [n_rows, L_B] -> float32 [n_rows, D]."""
        assert tokens.dtype == self.torch.int32 and tokens.is_cuda and tokens.is_contiguous()
        n = tokens.numel() // self.cfg.block_len
        out = self.torch.empty(n, self.cfg.d_model, dtype=self.torch.float32, device=self.device)
        with self._ordered():
            self._chk(lib.bt_embed(self.h, tokens.data_ptr(), n, out.data_ptr()))
        return out

    def bt_set_profile(self, on):
        self._chk(lib.bt_set_profile(self.h, int(on)))

    def bt_reset_profile(self):
        with self._ordered():
            self._chk(lib.bt_reset_profile(self.h))

    def bt_get_stats(self) -> bt_stats:
        st = bt_stats()
        with self._ordered():
            self._chk(lib.bt_get_stats(self.h, C.byref(st)))
        return st

    def close(self):
        if self.h:
            self.stream.synchronize()       # the workspace goes back to torch's allocator after this
            lib.bt_destroy(self.h)
            self.h = _P()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def probe_read(src, stream, out):
    """bt_probe_read on torch tensors: src uint8 (numel a multiple of PROBE_READ_GRAIN), out float32 scratch."""
    rc = lib.bt_probe_read(src.data_ptr(), src.numel(), stream.cuda_stream, out.data_ptr())
    if rc:
        raise BTError(rc, "bt_probe_read")


def probe_mfma(iters, random_operands, stream, out):
    rc = lib.bt_probe_mfma(int(iters), int(random_operands), stream.cuda_stream, out.data_ptr())
    if rc:
        raise BTError(rc, "bt_probe_mfma")

