"""ctypes binding of libladder.so (the C-ABI declared in include/ladder.h).

Argument marshalling only: every step of the forward runs in the HIP kernels of
the library.  PyTorch tensors are used as device memory (``data_ptr()``) and
for the stream handle.  Loading fails loudly when the library has not been
built (run ``python -c "import __graft_entry__ as g; g.build()"``); there is no
fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libladder.so")

LADDER_FP32, LADDER_BF16 = 0, 1
LADDER_WIRING_LADDER, LADDER_WIRING_STANDARD, LADDER_WIRING_PARALLEL = 0, 1, 2
LADDER_PATH_AUTO, LADDER_PATH_GENERIC = 0, 1
LADDER_OK, LADDER_E_ARG, LADDER_E_SHAPE, LADDER_E_STATE, LADDER_E_OVERFLOW, LADDER_E_HIP = 0, -1, -2, -3, -4, -5
(LADDER_K_REDUCE_NORM, LADDER_K_GEMV, LADDER_K_GEMM, LADDER_K_ROPE_APPEND, LADDER_K_ATTN_DECODE,
 LADDER_K_ATTN_PREFILL, LADDER_K_GENERIC, LADDER_K_OTHER, LADDER_K_FUSED_DECODE, LADDER_K_COUNT) = range(10)
KERNEL_CLASS_NAMES = ["reduce_norm", "gemv", "gemm", "rope_append", "attn_decode", "attn_prefill", "generic", "other", "fused_decode"]


class ladder_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "inter", "tp_degree", "n_real_shards",
        "max_batch", "max_seq", "max_tokens", "dtype", "wiring", "n_standard_layers", "reduce_on_side_stream",
        "peer_pool", "peer_rows", "kernel_path", "overlap_modules", "decode_graph", "decode_fused",
        "reduce_delay_us")] + [("rms_eps", C.c_float), ("rope_theta", C.c_float)]


class ladder_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in (
        "attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down")]


EXPORTS = {
    "ladder_init": (C.c_int, [C.POINTER(ladder_config), C.c_void_p, C.POINTER(C.c_void_p)]),
    "ladder_load_layer": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(ladder_layer_weights)]),
    "ladder_set_peer_partials": (C.c_int, [C.c_void_p, C.c_void_p]),
    "ladder_load_kv": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32]),
    "ladder_prefill": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]),
    "ladder_decode_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "ladder_prefill_stage": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "ladder_decode_step_stage": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "ladder_free": (None, [C.c_void_p]),
    "ladder_last_error": (C.c_char_p, [C.c_void_p]),
    "ladder_position": (C.c_int, [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "ladder_device_bytes": (C.c_size_t, [C.c_void_p]),
    "ladder_workspace_bytes": (C.c_size_t, [C.POINTER(ladder_config)]),
    "ladder_weight_bytes": (C.c_size_t, [C.POINTER(ladder_config)]),
    "ladder_set_wait_limit": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32]),
    "ladder_profile_enable": (C.c_int, [C.c_void_p, C.c_int32]),
    "ladder_profile_read": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_double)]),
    "ladder_profile_reset": (C.c_int, [C.c_void_p]),
    "ladder_calibration_copy": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t]),
    "ladder_timeline_enable": (C.c_int, [C.c_void_p, C.c_int32]),
    "ladder_timeline_read": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.POINTER(C.c_int64), C.POINTER(C.c_double)]),
    "ladder_load_head": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32]),
    "ladder_embed": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]),
    "ladder_head": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]),
    "ladder_head_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]),
}

_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it is not there (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                               "(hipcc --offload-arch=gfx950); there is no fallback path")
        handle = C.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def workspace_bytes(cfg: ladder_config) -> int:
    """Device bytes ladder_init(cfg) allocates apart from the weight store (host only)."""
    return int(lib().ladder_workspace_bytes(C.byref(cfg)))


def weight_bytes(cfg: ladder_config) -> int:
    """Device bytes of the weight store of ladder_init(cfg) (host only)."""
    return int(lib().ladder_weight_bytes(C.byref(cfg)))


class LadderError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"ladder error {code}: {text}")
        self.code = code


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def make_config(**kw) -> ladder_config:
    cfg = ladder_config()
    defaults = dict(tp_degree=1, n_real_shards=1, dtype=LADDER_BF16, wiring=LADDER_WIRING_LADDER,
                    n_standard_layers=0, reduce_on_side_stream=1, peer_pool=0, peer_rows=0,
                    kernel_path=LADDER_PATH_AUTO, overlap_modules=1, decode_graph=0, decode_fused=3, reduce_delay_us=0,
                    rms_eps=1e-5, rope_theta=1e4)
    defaults.update(kw)
    known = {n for n, _ in ladder_config._fields_}
    for k, v in defaults.items():
        if k not in known:
            raise KeyError(k)
        setattr(cfg, k, v)
    return cfg


def config_for(w, **override) -> ladder_config:
    """ladder_config of a seeded workload (paper_2501_06589_amd.inputs.Workload)."""
    kw = dict(n_layers=w.n_layers, hidden=w.hidden, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads,
              head_dim=w.head_dim, inter=w.inter, tp_degree=w.tp_degree, n_real_shards=w.n_real_shards,
              max_batch=w.batch, max_seq=w.max_seq, max_tokens=max(w.prefill, 1),
              dtype=LADDER_FP32 if w.dtype == "fp32" else LADDER_BF16,
              peer_pool=w.peer_pool if w.n_peers else 0,
              peer_rows=w.batch * max(w.prefill, 1) if w.n_peers else 0,
              rms_eps=w.rms_eps, rope_theta=w.rope_theta)
    kw.update(override)
    return make_config(**kw)


class Ladder:
    """Owner of one ladder_ctx.  Methods carry the C entry points' names without the prefix."""

    def __init__(self, cfg: ladder_config, stream: Optional[int] = None):
        import torch
        self._lib = lib()
        self.cfg = cfg
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        h = C.c_void_p()
        rc = self._lib.ladder_init(C.byref(cfg), C.c_void_p(stream), C.byref(h))
        if rc != LADDER_OK:
            raise LadderError(rc, (self._lib.ladder_last_error(None) or b"").decode())
        self._h = h
        self._keep = []          # tensors the library references without copying (peers)

    # -- error helper
    def _check(self, rc: int):
        if rc != LADDER_OK:
            raise LadderError(rc, (self._lib.ladder_last_error(self._h) or b"").decode())

    # -- the C side takes raw device pointers and cannot know how large the buffers behind them are:
    #    sizes, storage type, device and contiguity are checked here, where the tensors are still tensors
    def _want(self, name: str, t, numel: int, storage: bool = True):
        import torch
        if t is None:
            raise ValueError(f"{name} is missing")
        dt = (torch.float32 if self.cfg.dtype == LADDER_FP32 else torch.bfloat16) if storage else torch.float32
        if not t.is_cuda or not t.is_contiguous() or t.dtype != dt or t.numel() != numel:
            raise ValueError(f"{name}: need a contiguous {dt} device tensor of {numel} elements, got "
                             f"{tuple(t.shape)} {t.dtype} on {t.device}")

    def load_layer(self, layer: int, shard: int, tensors: Dict[str, "object"]):
        g = self.cfg
        nqd, nkvd = g.n_q_heads * g.head_dim, g.n_kv_heads * g.head_dim
        sizes = dict(attn_norm=g.hidden, wq=g.hidden * nqd, wk=g.hidden * nkvd, wv=g.hidden * nkvd, wo=nqd * g.hidden,
                     mlp_norm=g.hidden, w_gate=g.hidden * g.inter, w_up=g.hidden * g.inter, w_down=g.inter * g.hidden)
        w = ladder_layer_weights()
        for name, _ in ladder_layer_weights._fields_:
            self._want(name, tensors.get(name), sizes[name])
            setattr(w, name, _ptr(tensors[name]))
        self._check(self._lib.ladder_load_layer(self._h, layer, shard, C.byref(w)))

    def set_peer_partials(self, peers):
        g = self.cfg
        n = g.peer_pool * (g.tp_degree - g.n_real_shards) * g.peer_rows * g.hidden
        if peers is not None and n > 0:      # a configuration without peers: the library reports the misuse
            self._want("peers", peers, n)
        self._keep = [peers]
        self._check(self._lib.ladder_set_peer_partials(self._h, _ptr(peers)))

    def load_kv(self, layer: int, shard: int, k, v):
        g = self.cfg
        b, _, s, _ = k.shape
        k, v = k.contiguous(), v.contiguous()
        self._want("k", k, b * g.n_kv_heads * s * g.head_dim)
        self._want("v", v, b * g.n_kv_heads * s * g.head_dim)
        self._check(self._lib.ladder_load_kv(self._h, layer, shard, _ptr(k), _ptr(v), b, s))

    def prefill(self, x_in, x_out=None):
        import torch
        b, t, h = x_in.shape
        self._want("x_in", x_in, b * t * self.cfg.hidden)
        if x_out is None:
            x_out = torch.empty((b, t, h), dtype=torch.float32, device=x_in.device)
        self._want("x_out", x_out, b * t * self.cfg.hidden, storage=False)
        self._check(self._lib.ladder_prefill(self._h, _ptr(x_in), b, t, _ptr(x_out)))
        return x_out

    def decode_step(self, x_in, x_out=None):
        import torch
        _, batch = self.position()
        self._want("x_in", x_in, max(batch, 1) * self.cfg.hidden)
        if x_out is None:
            x_out = torch.empty(x_in.shape, dtype=torch.float32, device=x_in.device)
        self._want("x_out", x_out, max(batch, 1) * self.cfg.hidden, storage=False)
        self._check(self._lib.ladder_decode_step(self._h, _ptr(x_in), _ptr(x_out)))
        return x_out

    # -- pipeline stages: (residual, attn_out, mlp_out) in, the same three out
    def _stage_io(self, handoff, n):
        import torch
        res, att, mlp = handoff
        self._want("residual_in", res, n, storage=False)
        for name, t in (("attn_in", att), ("mlp_in", mlp)):
            if t is not None:
                self._want(name, t, n, storage=False)
        outs = tuple(torch.empty(res.shape, dtype=torch.float32, device=res.device) for _ in range(3))
        return (res, att, mlp), outs

    def prefill_stage(self, handoff):
        """handoff: (residual, attn_out, mlp_out), f32 device [B][T][H]; attn_out / mlp_out may be None (first stage)."""
        b, t, _ = handoff[0].shape
        ins, outs = self._stage_io(handoff, b * t * self.cfg.hidden)
        self._check(self._lib.ladder_prefill_stage(self._h, *[_ptr(x) for x in ins], b, t, *[_ptr(x) for x in outs]))
        return outs

    def decode_step_stage(self, handoff):
        _, batch = self.position()
        ins, outs = self._stage_io(handoff, max(batch, 1) * self.cfg.hidden)
        self._check(self._lib.ladder_decode_step_stage(self._h, *[_ptr(x) for x in ins], *[_ptr(x) for x in outs]))
        return outs

    # -- generation head
    def load_head(self, table, final_norm, w_lm):
        vocab, vocab_local = table.shape[0], w_lm.shape[1]
        self._want("table", table, vocab * self.cfg.hidden)
        self._want("final_norm", final_norm, self.cfg.hidden)
        self._want("w_lm", w_lm, self.cfg.hidden * vocab_local)
        self._check(self._lib.ladder_load_head(self._h, _ptr(table), _ptr(final_norm), _ptr(w_lm), vocab, vocab_local))
        self._vocab_local = vocab_local

    def embed(self, tokens):
        """tokens: int32 device tensor of any shape [...]; returns the embeddings [..., H] in the storage type."""
        import torch
        if not tokens.is_cuda or not tokens.is_contiguous() or tokens.dtype != torch.int32:
            raise ValueError("tokens: need a contiguous int32 device tensor")
        dt = torch.float32 if self.cfg.dtype == LADDER_FP32 else torch.bfloat16
        out = torch.empty(tuple(tokens.shape) + (self.cfg.hidden,), dtype=dt, device=tokens.device)
        self._check(self._lib.ladder_embed(self._h, _ptr(tokens), tokens.numel(), _ptr(out)))
        return out

    def head(self, x, want_logits=True):
        """x: f32 device [rows][H]; returns (logits f32 [rows][vocab_local] or None, tokens int32 [rows])."""
        import torch
        rows = x.shape[0]
        self._want("x", x, rows * self.cfg.hidden, storage=False)
        logits = torch.empty((rows, self._vocab_local), dtype=torch.float32, device=x.device) if want_logits else None
        toks = torch.empty((rows,), dtype=torch.int32, device=x.device)
        self._check(self._lib.ladder_head(self._h, _ptr(x), rows, _ptr(logits), _ptr(toks)))
        return logits, toks

    def head_static(self, x, tokens_out):
        """ladder_head_static: greedy tokens into the caller's int32 device tensor [rows]; allocates nothing."""
        import torch
        rows = x.shape[0]
        self._want("x", x, rows * self.cfg.hidden, storage=False)
        if not tokens_out.is_cuda or not tokens_out.is_contiguous() or tokens_out.dtype != torch.int32 or tokens_out.numel() != rows:
            raise ValueError("tokens_out: need a contiguous int32 device tensor of `rows` elements")
        self._check(self._lib.ladder_head_static(self._h, _ptr(x), rows, _ptr(tokens_out)))
        return tokens_out

    def position(self) -> Tuple[int, int]:
        p, b = C.c_int32(), C.c_int32()
        self._check(self._lib.ladder_position(self._h, C.byref(p), C.byref(b)))
        return p.value, b.value

    def device_bytes(self) -> int:
        return int(self._lib.ladder_device_bytes(self._h))

    def set_wait_limit(self, max_polls: int, target_bias: int):
        self._check(self._lib.ladder_set_wait_limit(self._h, max_polls, target_bias))

    def timeline_enable(self, on: bool):
        """Chained decode steps record, per persistent workgroup and block, when it was taken, ready and done."""
        self._check(self._lib.ladder_timeline_enable(self._h, 1 if on else 0))

    def timeline(self):
        """Records of the last chained step: (numpy structured array, clock ticks per microsecond)."""
        import numpy as np
        dt = np.dtype([("slot", "<i4"), ("launch", "<i4"), ("kind", "<i4"), ("tiles", "<i4"), ("weight_bytes", "<i8"),
                       ("t_take", "<u8"), ("t_ready", "<u8"), ("t_end", "<u8")])
        n, rate = C.c_int64(0), C.c_double(0.0)
        self._check(self._lib.ladder_timeline_read(self._h, None, 0, C.byref(n), C.byref(rate)))
        out = np.zeros(n.value, dtype=dt)
        self._check(self._lib.ladder_timeline_read(self._h, out.ctypes.data, n.value, C.byref(n), C.byref(rate)))
        return out, rate.value

    def profile_enable(self, on: bool):
        self._check(self._lib.ladder_profile_enable(self._h, 1 if on else 0))

    def profile_reset(self):
        self._check(self._lib.ladder_profile_reset(self._h))

    def calibration_copy(self, dst, src):
        """Plain copy kernel over two same-sized device tensors (the known-size dispatch HBM counters are scaled by)."""
        nbytes = src.numel() * src.element_size()
        if dst.numel() * dst.element_size() != nbytes:
            raise ValueError("calibration_copy: sizes differ")
        self._check(self._lib.ladder_calibration_copy(self._h, C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()),
                                                      C.c_size_t(nbytes)))

    def profile_read(self) -> Dict[str, Tuple[int, float]]:
        out = {}
        for cls, name in enumerate(KERNEL_CLASS_NAMES):
            n, ms = C.c_int64(), C.c_double()
            self._check(self._lib.ladder_profile_read(self._h, cls, C.byref(n), C.byref(ms)))
            out[name] = (n.value, ms.value)
        return out

    def free(self):
        if getattr(self, "_h", None) is not None and self._h:
            self._lib.ladder_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass
