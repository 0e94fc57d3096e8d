"""ctypes binding of libl2pd.so: argument marshalling only.

Every step of the decoding path runs in the library's HIP kernels; torch is used for device
memory (tensors whose ``data_ptr()`` is handed over) and for the stream.  If the library has not
been built, importing this module raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import torch

from . import synth

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libl2pd.so")

L2PD_OK, L2PD_EINVAL, L2PD_ENOMEM, L2PD_EHIP, L2PD_ENOTIMPL = 0, -1, -2, -3, -4
K_NONE, K_GEMM_QKV, K_GEMM_O, K_GEMM_GATEUP, K_GEMM_DOWN, K_ATTN, K_LMHEAD, K_NORM, K_UPDATE = range(9)


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab",
                                         "mask_id", "eos_id")] + \
               [("rope_base", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int32)]


class Weights(C.Structure):
    _fields_ = [("tok_emb_dev", C.c_void_p), ("lm_head_dev", C.c_void_p), ("final_norm_g_dev", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("attn_norm_g", "wq", "wk", "wv", "wo", "ffn_norm_g",
                                                       "w_gate", "w_up", "w_down")]


FILTER_MAX_LAYERS = 4


class Filter(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("in_dim", C.c_int32), ("hidden", C.c_int32),
                ("w_dev", C.c_void_p * FILTER_MAX_LAYERS), ("b_dev", C.c_void_p * FILTER_MAX_LAYERS)]


def filter_layers(flt: Dict[str, torch.Tensor]):
    """[(w1, b1), ..., (wN, bN)] of a filter given as a dict with those keys."""
    out = []
    while f"w{len(out) + 1}" in flt:
        k = len(out) + 1
        out.append((flt[f"w{k}"], flt[f"b{k}"]))
    if not 1 <= len(out) <= FILTER_MAX_LAYERS or len(flt) != 2 * len(out):
        raise ValueError("a filter is {w1, b1, ..., wN, bN} with 1 <= N <= 4")
    return out


def _filter_struct(flt: Dict[str, torch.Tensor]) -> Filter:
    layers = filter_layers(flt)
    in_dim = layers[0][0].shape[1]
    hidden = layers[0][0].shape[0] if len(layers) > 1 else 0
    for k, (w, b) in enumerate(layers):
        want = (in_dim if k == len(layers) - 1 else hidden, in_dim if k == 0 else hidden)
        if tuple(w.shape) != want or tuple(b.shape) != want[:1]:
            raise ValueError(f"filter layer {k + 1}: expected weight {want}, got {tuple(w.shape)} / {tuple(b.shape)}")
    f = Filter(len(layers), in_dim, hidden)
    for k, (w, b) in enumerate(layers):
        f.w_dev[k] = w.data_ptr()
        f.b_dev[k] = b.data_ptr()
    return f


class LogitBias(C.Structure):
    _fields_ = [("token_id", C.c_int32), ("gen_pos_from", C.c_int32), ("value", C.c_float)]


CACHE_NONE, CACHE_PREFIX, CACHE_DUAL = 0, 1, 2
EOTP_OFF, EOTP_BLOCK, EOTP_STEP = 0, 1, 2
RAGGED_OFF, RAGGED_BLOCKS, RAGGED_COMPACT = 0, 1, 2


class DecodeCfg(C.Structure):
    _fields_ = [("gen_len", C.c_int32), ("block_len", C.c_int32), ("threshold", C.c_float), ("eotp", C.c_int32),
                ("kv_cache", C.c_int32), ("keep_kv", C.c_int32), ("ragged", C.c_int32), ("bias", LogitBias)]


class TrainCfg(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("epochs", C.c_int32)]


EXPORTS = ("l2pd_workspace_bytes", "l2pd_create", "l2pd_destroy", "l2pd_forward", "l2pd_denoise_step",
           "l2pd_generate", "l2pd_egp_rollout", "l2pd_filter_train", "l2pd_filter_train_static", "l2pd_profile_select", "l2pd_profile_read", "l2pd_generate_stats", "l2pd_strerror")


def load_library() -> C.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it first "
                          "(python -c 'import __graft_entry__ as g; g.build()')")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.l2pd_workspace_bytes.restype = sz
    lib.l2pd_workspace_bytes.argtypes = [C.POINTER(ModelDesc), i32, i32, i32]
    lib.l2pd_create.restype = i32
    lib.l2pd_create.argtypes = [C.POINTER(ModelDesc), C.POINTER(Weights), i32, i32, i32, vp, sz, C.POINTER(vp)]
    lib.l2pd_destroy.restype = None
    lib.l2pd_destroy.argtypes = [vp]
    lib.l2pd_forward.restype = i32
    lib.l2pd_forward.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp]
    lib.l2pd_denoise_step.restype = i32
    lib.l2pd_denoise_step.argtypes = [vp, vp, i32, i32, C.POINTER(DecodeCfg), C.POINTER(Filter), vp,
                                      vp, vp, vp, vp, vp, vp]
    lib.l2pd_generate.restype = i32
    lib.l2pd_generate.argtypes = [vp, vp, i32, i32, C.POINTER(DecodeCfg), C.POINTER(Filter), vp, vp, vp, vp]
    lib.l2pd_egp_rollout.restype = i32
    lib.l2pd_egp_rollout.argtypes = [vp, vp, vp, i32, i32, C.POINTER(DecodeCfg), vp, vp, vp, vp]
    lib.l2pd_filter_train.restype = i32
    lib.l2pd_filter_train.argtypes = [C.POINTER(Filter), vp, vp, C.c_int64, C.POINTER(TrainCfg), vp, vp, vp]
    lib.l2pd_filter_train_static.restype = i32
    lib.l2pd_filter_train_static.argtypes = [C.POINTER(Filter), vp, vp, C.c_int64, C.POINTER(TrainCfg), vp, vp]
    lib.l2pd_profile_select.restype = i32
    lib.l2pd_profile_select.argtypes = [vp, i32]
    lib.l2pd_profile_read.restype = i32
    lib.l2pd_profile_read.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_double)]
    lib.l2pd_generate_stats.restype = i32
    lib.l2pd_generate_stats.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    lib.l2pd_strerror.restype = C.c_char_p
    lib.l2pd_strerror.argtypes = [i32]
    return lib


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = load_library()
    return _lib


class L2PDError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().l2pd_strerror(status).decode()} ({status})")


def _check(status: int, where: str):
    if status != L2PD_OK:
        raise L2PDError(status, where)


def model_desc(m: synth.ModelShape) -> ModelDesc:
    return ModelDesc(m.n_layers, m.d_model, m.n_heads, m.head_dim, m.d_ffn, m.vocab, m.mask_id, m.eos_id,
                     m.rope_base, m.rms_eps, 0 if m.dtype == "fp32" else 1)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class Engine:
    """A model resident in HBM plus a library context.  Tensors in, tensors out."""

    def __init__(self, shape: synth.ModelShape, weights: Dict[str, torch.Tensor], max_batch: int, max_seq: int,
                 prefix_cache: bool = False):
        """`prefix_cache`: allocate the per-layer K/V stores that the cached decode modes (prefix or dual) need."""
        self.shape = shape
        self.weights = weights          # keeps the device tensors alive
        self.max_batch, self.max_seq, self.prefix_cache = max_batch, max_seq, prefix_cache
        self._desc = model_desc(shape)
        L = shape.n_layers
        arr = lambda name: (C.c_void_p * L)(*[weights[f"layers.{l}.{name}"].data_ptr() for l in range(L)])
        self._arrays = {n: arr(n) for n in ("attn_norm_g", "wq", "wk", "wv", "wo", "ffn_norm_g", "w_gate",
                                            "w_up", "w_down")}
        w = Weights(weights["tok_emb"].data_ptr(), weights["lm_head"].data_ptr(),
                    weights["final_norm_g"].data_ptr(),
                    *[C.cast(self._arrays[n], C.POINTER(C.c_void_p)) for n in
                      ("attn_norm_g", "wq", "wk", "wv", "wo", "ffn_norm_g", "w_gate", "w_up", "w_down")])
        nbytes = lib().l2pd_workspace_bytes(C.byref(self._desc), max_batch, max_seq, int(prefix_cache))
        if nbytes == 0:
            raise L2PDError(L2PD_EINVAL, "l2pd_workspace_bytes")
        dev = weights["tok_emb"].device
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        self._ctx = C.c_void_p()
        _check(lib().l2pd_create(C.byref(self._desc), C.byref(w), max_batch, max_seq, int(prefix_cache),
                                 self.workspace.data_ptr(), nbytes, C.byref(self._ctx)), "l2pd_create")

    def close(self):
        if getattr(self, "_ctx", None) is not None and self._ctx.value:
            lib().l2pd_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- marshalling helpers ----
    @staticmethod
    def filter_struct(flt: Dict[str, torch.Tensor]) -> Filter:
        return _filter_struct(flt)

    @staticmethod
    def cfg_struct(gen_len, block_len, threshold, eotp=False, prefix_cache=False, bias=None,
                   dual_cache=False, ragged=False) -> DecodeCfg:
        b = LogitBias(0, 0, 0.0) if bias is None else LogitBias(int(bias[0]), int(bias[1]), float(bias[2]))
        if prefix_cache and dual_cache:
            raise ValueError("prefix_cache and dual_cache are alternatives")
        return DecodeCfg(gen_len, block_len, threshold, int(eotp), CACHE_DUAL if dual_cache else int(bool(prefix_cache)), 0, int(ragged), b)

    # ---- entry points ----
    def forward(self, tokens: torch.Tensor, row_begin: int = 0, row_count: Optional[int] = None) -> torch.Tensor:
        B, T = tokens.shape
        if row_count is None:
            row_count = T - row_begin
        out = torch.empty((B, max(row_count, 0), self.shape.vocab), dtype=torch.float32, device=tokens.device)
        _check(lib().l2pd_forward(self._ctx, tokens.data_ptr(), B, T, row_begin, row_count, out.data_ptr(),
                                  _stream()), "l2pd_forward")
        return out

    def denoise_step(self, tokens: torch.Tensor, prompt_len: int, state: torch.Tensor, flt, cfg: DecodeCfg,
                     want_logits: bool = False):
        """Runs one step in place on (tokens, state); returns the taps as a dict of tensors."""
        B = tokens.shape[0]
        s, dev = cfg.block_len, tokens.device
        taps = dict(conf=torch.empty((B, s), dtype=torch.float32, device=dev),
                    pred=torch.empty((B, s), dtype=torch.int32, device=dev),
                    p=torch.empty((B, s), dtype=torch.float32, device=dev),
                    sel=torch.zeros((B, s), dtype=torch.uint8, device=dev))
        logits = torch.empty((B, s, self.shape.vocab), dtype=torch.float32, device=dev) if want_logits else None
        f = self.filter_struct(flt)
        _check(lib().l2pd_denoise_step(self._ctx, tokens.data_ptr(), B, prompt_len, C.byref(cfg), C.byref(f),
                                       state.data_ptr(), _ptr(logits), taps["conf"].data_ptr(),
                                       taps["pred"].data_ptr(), taps["p"].data_ptr(), taps["sel"].data_ptr(),
                                       _stream()), "l2pd_denoise_step")
        if want_logits:
            taps["logits"] = logits
        return taps

    def generate(self, prompt: torch.Tensor, flt, cfg: DecodeCfg):
        """Returns (tokens [B, gen_len], steps [B], decoded_len [B]) as device tensors."""
        B, P = prompt.shape
        dev = prompt.device
        tokens = torch.empty((B, cfg.gen_len), dtype=torch.int32, device=dev)
        steps = torch.empty((B,), dtype=torch.int32, device=dev)
        dlen = torch.empty((B,), dtype=torch.int32, device=dev)
        f = self.filter_struct(flt)
        _check(lib().l2pd_generate(self._ctx, prompt.data_ptr(), B, P, C.byref(cfg), C.byref(f),
                                   tokens.data_ptr(), steps.data_ptr(), dlen.data_ptr(), _stream()),
               "l2pd_generate")
        return tokens, steps, dlen

    def egp_rollout(self, prompt: torch.Tensor, reference: torch.Tensor, cfg: DecodeCfg):
        """EGP rollout against `reference` [B, gen_len] (int32).  Returns (conf_rows [B, gen_len, s],
        label_rows [B, gen_len, s], steps [B]); rows beyond steps[b] are zero."""
        B, P = prompt.shape
        dev = prompt.device
        conf = torch.zeros((B, cfg.gen_len, cfg.block_len), dtype=torch.float32, device=dev)
        label = torch.zeros_like(conf)
        steps = torch.empty((B,), dtype=torch.int32, device=dev)
        _check(lib().l2pd_egp_rollout(self._ctx, prompt.data_ptr(), reference.data_ptr(), B, P, C.byref(cfg),
                                      conf.data_ptr(), label.data_ptr(), steps.data_ptr(), _stream()),
               "l2pd_egp_rollout")
        return conf, label, steps

    def profile_select(self, kernel_class: int):
        _check(lib().l2pd_profile_select(self._ctx, kernel_class), "l2pd_profile_select")

    def profile_read(self):
        n, ms = C.c_int64(), C.c_double()
        _check(lib().l2pd_profile_read(self._ctx, C.byref(n), C.byref(ms)), "l2pd_profile_read")
        return n.value, ms.value

    def generate_stats(self):
        """(step launches, sum over them of the sequences each ran over) of the last generate."""
        steps, seq_steps = C.c_int64(), C.c_int64()
        _check(lib().l2pd_generate_stats(self._ctx, C.byref(steps), C.byref(seq_steps)), "l2pd_generate_stats")
        return steps.value, seq_steps.value


def train_filter(flt: Dict[str, torch.Tensor], conf_rows: torch.Tensor, label_rows: torch.Tensor, epochs: int,
                 lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, losses: Optional[torch.Tensor] = None,
                 static_scratch: bool = False):
    """Trains the filter IN PLACE (device fp32 tensors w1, b1, ..., wN, bN) on rows [n, s]; returns the
    per-epoch losses as a device tensor (`losses`, if given, receives them: [epochs] fp32 on the device).
    `static_scratch` takes l2pd_filter_train_static: no buffer is allocated here either when `losses` is given."""
    for t in list(flt.values()) + [conf_rows, label_rows]:
        if t.dtype != torch.float32 or not t.is_contiguous() or not t.is_cuda:
            raise ValueError("train_filter needs contiguous fp32 device tensors")
    f = _filter_struct(flt)
    s = f.in_dim
    n = conf_rows.shape[0]
    if conf_rows.shape != (n, s) or label_rows.shape != (n, s):
        raise ValueError("rows must be [n, in_dim]")
    tc = TrainCfg(lr, beta1, beta2, eps, weight_decay, epochs)
    if losses is None:
        losses = torch.empty(epochs, dtype=torch.float32, device=conf_rows.device)
    if static_scratch:
        _check(lib().l2pd_filter_train_static(C.byref(f), conf_rows.data_ptr(), label_rows.data_ptr(), n, C.byref(tc),
                                              losses.data_ptr(), _stream()), "l2pd_filter_train_static")
        return losses
    n_params = sum(t.numel() for t in flt.values())
    state = torch.empty(2 * n_params, dtype=torch.float32, device=conf_rows.device)
    _check(lib().l2pd_filter_train(C.byref(f), conf_rows.data_ptr(), label_rows.data_ptr(), n, C.byref(tc),
                                   state.data_ptr(), losses.data_ptr(), _stream()), "l2pd_filter_train")
    return losses


def engine_for(w: synth.Workload, seed: int, device="cuda", max_batch: Optional[int] = None,
               lm_head_scale: float = 1.0) -> Engine:
    weights = synth.make_weights(w.model, seed, device, lm_head_scale=lm_head_scale)
    return Engine(w.model, weights, max_batch or w.batch, w.prompt_len + w.gen_len, w.prefix_cache or w.dual_cache)
