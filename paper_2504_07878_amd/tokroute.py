"""Thin Python binding of libtokroute (the C ABI in include/tokroute.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels. PyTorch is used for
device memory (weights, workspace, output buffers) and for the current stream handle. There is no CPU
fallback: if the library is missing or no GPU is present, calls raise.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libtokroute.so")

OK, ERR_INVALID_ARG, ERR_SHAPE, ERR_CAPACITY, ERR_STATE, ERR_HIP = 0, -1, -2, -3, -4, -5
F32, BF16 = 0, 1
JOINT, SMALL_ONLY = 0, 1
ROUTE_IF_BELOW, ROUTE_IF_ABOVE = 0, 1
POLICY_MLP, POLICY_CONFIDENCE, POLICY_LINEAR = 0, 1, 2
POST_FINAL_NORM, PRE_FINAL_NORM = 0, 1
KERNEL_FAMILIES = ("setup", "prep", "qkv", "attention", "oproj", "gateup", "down", "lmhead", "tail_merge", "qkv_attention")   # TR_KERNEL_*

EXPORTS = ["tr_workspace_bytes", "tr_create", "tr_destroy", "tr_prefill", "tr_decode_step", "tr_decode_step_dev", "tr_decode_step_active", "tr_extend", "tr_tail", "tr_tail_noalloc", "tr_set_threshold",
           "tr_set_mode", "tr_seq_len", "tr_seq_truncate", "tr_seq_fork", "tr_seq_load_kv", "tr_counters_ptr", "tr_profile_enable", "tr_profile_select",
           "tr_profile_read", "tr_profile_chain", "tr_last_error"]


class tr_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + [
        ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("dtype", C.c_int32), ("kv_dtype", C.c_int32),
        ("tie_lm_head", C.c_int32), ("router_hidden", C.c_int32), ("threshold", C.c_float), ("route_dir", C.c_int32),
        ("hidden_tap", C.c_int32), ("max_batch", C.c_int32), ("max_seq", C.c_int32), ("route_policy", C.c_int32),
        ("kv_page", C.c_int32), ("kv_pool_pages", C.c_int32)]


_PP = C.POINTER(C.c_void_p)


class tr_weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + [
        (n, _PP) for n in ("ln1", "wq", "wk", "wv", "bq", "bk", "bv", "wo", "ln2", "wg", "wu", "wd")] + [
        (n, C.c_void_p) for n in ("r_w1", "r_b1", "r_w2", "r_b2")]


class tr_out(C.Structure):
    _fields_ = [("token", C.c_void_p), ("conf", C.c_void_p), ("score", C.c_void_p), ("flag", C.c_void_p),
                ("hidden", C.c_void_p), ("logits", C.c_void_p)]


_lib = None


def load_library():
    """Load libtokroute.so and declare its entry points. Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2504_07878_amd.build` (or __graft_entry__.build())")
        L = C.CDLL(LIB_PATH)
        vp, i32, f32 = C.c_void_p, C.c_int32, C.c_float
        L.tr_workspace_bytes.argtypes = [C.POINTER(tr_config)]; L.tr_workspace_bytes.restype = C.c_size_t
        L.tr_create.argtypes = [C.POINTER(tr_config), C.POINTER(tr_weights), vp, C.c_size_t, C.POINTER(vp)]
        L.tr_destroy.argtypes = [vp]; L.tr_destroy.restype = None
        L.tr_prefill.argtypes = [vp, vp, i32, vp, vp, vp, C.POINTER(tr_out)]
        L.tr_extend.argtypes = [vp, vp, i32, vp, vp, vp, C.POINTER(tr_out)]
        L.tr_decode_step.argtypes = [vp, vp, i32, vp, vp, C.POINTER(tr_out)]
        L.tr_decode_step_dev.argtypes = [vp, vp, i32, vp, vp, C.POINTER(tr_out)]
        L.tr_decode_step_active.argtypes = [vp, vp, i32, vp, vp, vp, i32, vp, vp, C.POINTER(tr_out)]
        L.tr_tail.argtypes = [vp, vp, i32, vp, C.POINTER(tr_out)]
        L.tr_tail_noalloc.argtypes = [vp, vp, i32, vp, C.POINTER(tr_out)]
        L.tr_set_threshold.argtypes = [vp, f32]
        L.tr_set_mode.argtypes = [vp, i32]
        L.tr_seq_len.argtypes = [vp, i32, C.POINTER(i32)]
        L.tr_seq_truncate.argtypes = [vp, i32, i32]
        L.tr_seq_fork.argtypes = [vp, vp, i32, i32]
        L.tr_seq_load_kv.argtypes = [vp, vp, i32, i32, vp, vp]
        L.tr_counters_ptr.argtypes = [vp, C.POINTER(vp)]
        L.tr_profile_enable.argtypes = [vp, i32]
        L.tr_profile_select.argtypes = [vp, i32]
        L.tr_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.tr_profile_chain.argtypes = [vp, vp, i32, i32]
        L.tr_last_error.argtypes = [vp]; L.tr_last_error.restype = C.c_char_p
        _lib = L
    return _lib


class TokrouteError(RuntimeError):
    def __init__(self, code, what, detail=""):
        super().__init__(f"{what}: error {code} {detail}")
        self.code = code


def to_device(a: np.ndarray, dtype: int, device="cuda:0") -> torch.Tensor:
    """numpy fp32 array or bf16 bit patterns (uint16) -> device tensor of the matching torch dtype."""
    if dtype == F32:
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device).view(torch.bfloat16)


class Outputs:
    """Device output buffers of one call (reusable across calls with the same n)."""

    def __init__(self, n, d, vocab, want_logits=False, want_hidden=True, device="cuda:0"):
        self.n = n
        self.token = torch.zeros(n, dtype=torch.int32, device=device)
        self.conf = torch.zeros(n, dtype=torch.float32, device=device)
        self.score = torch.zeros(n, dtype=torch.float32, device=device)
        self.flag = torch.zeros(n, dtype=torch.int32, device=device)
        self.hidden = torch.zeros((n, d), dtype=torch.float32, device=device) if want_hidden else None
        self.logits = torch.zeros((n, vocab), dtype=torch.float32, device=device) if want_logits else None
        self.struct = tr_out(self.token.data_ptr(), self.conf.data_ptr(), self.score.data_ptr(), self.flag.data_ptr(),
                             self.hidden.data_ptr() if want_hidden else None, self.logits.data_ptr() if want_logits else None)

    FIELDS = ("token", "conf", "score", "flag", "hidden", "logits")

    def cpu(self, fields=FIELDS, stream_only=False):
        """Synchronise and copy the named outputs (default: all) to numpy; the others are None.

        stream_only: wait for the current stream only (the one the outputs were produced on) instead of the whole device,
        so that work on other streams keeps running."""
        if not stream_only:
            torch.cuda.synchronize()
        o = type("HostOutputs", (), {})()
        for k in self.FIELDS:
            v = getattr(self, k) if k in fields else None
            setattr(o, k, None if v is None else v.cpu().numpy())
        return o


class Model:
    """A tr_ctx over device copies of numpy weights (dict name -> array; per-layer names ``l{i}.wq`` ...)."""

    def __init__(self, shape: dict, weights: dict, max_batch: int, max_seq: int, route_dir=ROUTE_IF_BELOW,
                 hidden_tap=POST_FINAL_NORM, device="cuda:0", route_policy=POLICY_MLP, kv_page=0, kv_pool_pages=0):
        if not torch.cuda.is_available():
            raise RuntimeError("tokroute needs a GPU: no CPU path exists")
        self.lib = load_library()
        self.device = device
        s = self.shape = dict(shape)
        self.cfg = tr_config(s["n_layers"], s["d_model"], s["n_q_heads"], s["n_kv_heads"], s["head_dim"], s["d_ffn"], s["vocab"],
                             s["rms_eps"], s["rope_theta"], s["dtype"], s["kv_dtype"], s["tie_lm_head"], s["router_hidden"],
                             s["threshold"], route_dir, hidden_tap, max_batch, max_seq, route_policy, kv_page, kv_pool_pages)
        dt, L = s["dtype"], s["n_layers"]
        self.dev = {k: (v if isinstance(v, torch.Tensor) else to_device(v, dt, device)) for k, v in weights.items()}
        self._arrs = []

        def one(name):
            t = self.dev.get(name)
            return None if t is None else t.data_ptr()

        def per_layer(name):
            if f"l0.{name}" not in self.dev:
                return None
            arr = (C.c_void_p * L)(*[self.dev[f"l{i}.{name}"].data_ptr() for i in range(L)])
            self._arrs.append(arr)
            return C.cast(arr, _PP)

        w = tr_weights(one("tok_emb"), one("lm_head"), one("final_norm"),
                       *[per_layer(n) for n in ("ln1", "wq", "wk", "wv", "bq", "bk", "bv", "wo", "ln2", "wg", "wu", "wd")],
                       one("r_w1"), one("r_b1"), one("r_w2"), one("r_b2"))
        nbytes = self.lib.tr_workspace_bytes(C.byref(self.cfg))
        if nbytes == 0:
            raise TokrouteError(ERR_SHAPE, "tr_workspace_bytes", "(configuration not supported)")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self._h = C.c_void_p()
        rc = self.lib.tr_create(C.byref(self.cfg), C.byref(w), self.workspace.data_ptr(), nbytes, C.byref(self._h))
        if rc:
            raise TokrouteError(rc, "tr_create")

    # -- helpers
    def _check(self, rc, what):
        if rc:
            raise TokrouteError(rc, what, (self.lib.tr_last_error(self._h) or b"").decode())

    @staticmethod
    def _stream():
        return torch.cuda.current_stream().cuda_stream

    def outputs(self, n, want_logits=False, want_hidden=True):
        return Outputs(n, self.shape["d_model"], self.shape["vocab"], want_logits, want_hidden, self.device)

    def close(self):
        if getattr(self, "_h", None):
            torch.cuda.synchronize()
            self.lib.tr_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the ABI, same names
    def prefill(self, slots, prompts, out: Outputs = None, want_logits=False):
        slots = np.ascontiguousarray(slots, dtype=np.int32)
        flat = np.ascontiguousarray(np.concatenate([np.asarray(p, dtype=np.int32) for p in prompts]), dtype=np.int32)
        offs = np.zeros(len(prompts) + 1, np.int32); offs[1:] = np.cumsum([len(p) for p in prompts])
        out = out or self.outputs(len(slots), want_logits)
        self._check(self.lib.tr_prefill(self._h, self._stream(), len(slots), slots.ctypes.data, flat.ctypes.data, offs.ctypes.data,
                                        C.byref(out.struct)), "tr_prefill")
        return out

    def extend(self, slots, segments, out: Outputs = None, want_logits=False):
        slots = np.ascontiguousarray(slots, dtype=np.int32)
        flat = np.ascontiguousarray(np.concatenate([np.asarray(p, dtype=np.int32) for p in segments]), dtype=np.int32)
        offs = np.zeros(len(segments) + 1, np.int32); offs[1:] = np.cumsum([len(p) for p in segments])
        out = out or self.outputs(len(slots), want_logits)
        self._check(self.lib.tr_extend(self._h, self._stream(), len(slots), slots.ctypes.data, flat.ctypes.data, offs.ctypes.data,
                                       C.byref(out.struct)), "tr_extend")
        return out

    def decode_step(self, slots, in_tokens, out: Outputs = None, want_logits=False):
        slots = np.ascontiguousarray(slots, dtype=np.int32)
        toks = np.ascontiguousarray(in_tokens, dtype=np.int32)
        if toks.shape != slots.shape:
            raise ValueError("slots and in_tokens differ in length")
        out = out or self.outputs(len(slots), want_logits)
        self._check(self.lib.tr_decode_step(self._h, self._stream(), len(slots), slots.ctypes.data, toks.ctypes.data,
                                            C.byref(out.struct)), "tr_decode_step")
        return out

    def decode_step_dev(self, slots, in_tokens: torch.Tensor, out: Outputs = None, want_logits=False):
        """Decode step whose input tokens are a device int32 tensor [n] (e.g. the `token` field of the previous outputs)."""
        slots = np.ascontiguousarray(slots, dtype=np.int32)
        assert in_tokens.is_cuda and in_tokens.dtype == torch.int32 and in_tokens.is_contiguous() and in_tokens.numel() == len(slots)
        out = out or self.outputs(len(slots), want_logits)
        self._check(self.lib.tr_decode_step_dev(self._h, self._stream(), len(slots), slots.ctypes.data, in_tokens.data_ptr(),
                                                C.byref(out.struct)), "tr_decode_step_dev")
        return out

    def decode_step_active(self, slots, flags: torch.Tensor, in_tokens: torch.Tensor, n_max: int, active: torch.Tensor,
                           next_tokens: torch.Tensor = None, out: Outputs = None, want_logits=False):
        """Decode step of the candidates (`slots`) whose device-side flag is set, at most n_max of them; see tr_decode_step_active.
        flags, in_tokens: device int32 [n]; active: device int32 [2 + n_max]; next_tokens: device int32 [n] or None."""
        slots = np.ascontiguousarray(slots, dtype=np.int32)
        for t, m in ((flags, len(slots)), (in_tokens, len(slots)), (active, 2 + n_max)) + (((next_tokens, len(slots)),) if next_tokens is not None else ()):
            assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous() and t.numel() == m
        out = out or self.outputs(n_max, want_logits)
        self._check(self.lib.tr_decode_step_active(self._h, self._stream(), len(slots), slots.ctypes.data, flags.data_ptr(), in_tokens.data_ptr(),
                                                   int(n_max), active.data_ptr(), None if next_tokens is None else next_tokens.data_ptr(),
                                                   C.byref(out.struct)), "tr_decode_step_active")
        return out

    def tail(self, x: torch.Tensor, out: Outputs = None, want_logits=False):
        """x: device fp32 [n][d_model] residual-stream rows."""
        assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.shape[1] == self.shape["d_model"]
        out = out or self.outputs(x.shape[0], want_logits)
        self._check(self.lib.tr_tail(self._h, self._stream(), x.shape[0], x.data_ptr(), C.byref(out.struct)), "tr_tail")
        return out

    def tail_noalloc(self, x: torch.Tensor, out: Outputs):
        """tr_tail with the library's static device scratch; `out` must exist already (nothing is allocated here)."""
        assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.shape[1] == self.shape["d_model"]
        self._check(self.lib.tr_tail_noalloc(self._h, self._stream(), x.shape[0], x.data_ptr(), C.byref(out.struct)), "tr_tail_noalloc")
        return out

    def set_threshold(self, t):
        self._check(self.lib.tr_set_threshold(self._h, float(t)), "tr_set_threshold")

    def set_mode(self, m):
        self._check(self.lib.tr_set_mode(self._h, int(m)), "tr_set_mode")

    def seq_len(self, slot):
        v = C.c_int32()
        self._check(self.lib.tr_seq_len(self._h, int(slot), C.byref(v)), "tr_seq_len")
        return v.value

    def seq_truncate(self, slot, new_len):
        self._check(self.lib.tr_seq_truncate(self._h, int(slot), int(new_len)), "tr_seq_truncate")

    def seq_fork(self, src, dst):
        self._check(self.lib.tr_seq_fork(self._h, self._stream(), int(src), int(dst)), "tr_seq_fork")

    def load_kv(self, slot, k: torch.Tensor, v: torch.Tensor):
        """k, v: device tensors [layer][kv_head][len][head_dim] in the cache storage type."""
        want = torch.float32 if self.shape["kv_dtype"] == F32 else torch.bfloat16
        assert k.is_cuda and v.is_cuda and k.dtype == want and v.dtype == want and k.is_contiguous() and v.is_contiguous()
        assert k.shape == v.shape and k.shape[0] == self.shape["n_layers"] and k.shape[1] == self.shape["n_kv_heads"]
        self._check(self.lib.tr_seq_load_kv(self._h, self._stream(), int(slot), k.shape[2], k.data_ptr(), v.data_ptr()), "tr_seq_load_kv")

    def counters(self):
        """Synchronise and return the [max_batch][2] int64 counters (n_generated, n_routed)."""
        p = C.c_void_p()
        self._check(self.lib.tr_counters_ptr(self._h, C.byref(p)), "tr_counters_ptr")
        off = p.value - self.workspace.data_ptr()
        n = self.cfg.max_batch * 2 * 8
        torch.cuda.synchronize()
        return self.workspace[off:off + n].cpu().numpy().view(np.int64).reshape(self.cfg.max_batch, 2).copy()

    def profile_enable(self, on=True):
        self._check(self.lib.tr_profile_enable(self._h, int(bool(on))), "tr_profile_enable")

    def profile_select(self, family: int):
        self._check(self.lib.tr_profile_select(self._h, int(family)), "tr_profile_select")

    def profile_read(self):
        ms, gap, n = C.c_double(), C.c_double(), C.c_int64()
        self._check(self.lib.tr_profile_read(self._h, C.byref(ms), C.byref(gap), C.byref(n)), "tr_profile_read")
        return ms.value, gap.value, n.value
