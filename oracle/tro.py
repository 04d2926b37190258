"""ctypes front end of the CPU oracle (``tro.c``). TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this. It never touches
the GPU library and the GPU library never touches it.

Arrays are numpy: fp32 tensors as float32, bf16 tensors as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libtro.so")

F32, BF16 = 0, 1
OK, ERR_INVALID_ARG, ERR_SHAPE, ERR_CAPACITY, ERR_STATE = 0, -1, -2, -3, -4
JOINT, SMALL_ONLY = 0, 1
ROUTE_IF_BELOW, ROUTE_IF_ABOVE = 0, 1
POLICY_MLP, POLICY_CONFIDENCE, POLICY_LINEAR = 0, 1, 2
POST_FINAL_NORM, PRE_FINAL_NORM = 0, 1


def build(force: bool = True) -> str:
    """Compile tro.c into libtro.so with gcc."""
    src = os.path.join(HERE, "tro.c")
    if force or not os.path.exists(LIB_PATH) or os.path.getmtime(LIB_PATH) < os.path.getmtime(src):
        cmd = ["gcc", "-O3", "-mavx2", "-mfma", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", LIB_PATH, src, "-lm"]
        subprocess.run(cmd, check=True)
    return LIB_PATH


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + [
        ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("dtype", C.c_int32), ("kv_dtype", C.c_int32),
        ("tie_lm_head", C.c_int32), ("router_hidden", C.c_int32), ("threshold", C.c_float), ("route_dir", C.c_int32),
        ("hidden_tap", C.c_int32), ("max_batch", C.c_int32), ("max_seq", C.c_int32), ("route_policy", C.c_int32)]


_PP = C.POINTER(C.c_void_p)


class Weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + [
        (n, _PP) for n in ("ln1", "wq", "wk", "wv", "bq", "bk", "bv", "wo", "ln2", "wg", "wu", "wd")] + [
        (n, C.c_void_p) for n in ("r_w1", "r_b1", "r_w2", "r_b2")]


class Out(C.Structure):
    _fields_ = [("token", C.c_void_p), ("conf", C.c_void_p), ("score", C.c_void_p), ("flag", C.c_void_p),
                ("hidden", C.c_void_p), ("logits", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            build()
        L = C.CDLL(LIB_PATH)
        vp, i32, f32 = C.c_void_p, C.c_int32, C.c_float
        L.tro_create.argtypes = [C.POINTER(Config), C.POINTER(Weights), C.POINTER(vp)]
        L.tro_destroy.argtypes = [vp]; L.tro_destroy.restype = None
        L.tro_prefill.argtypes = [vp, i32, vp, vp, vp, C.POINTER(Out)]
        L.tro_decode_step.argtypes = [vp, i32, vp, vp, C.POINTER(Out)]
        L.tro_extend.argtypes = [vp, i32, vp, vp, vp, C.POINTER(Out)]
        L.tro_seq_fork.argtypes = [vp, i32, i32]
        L.tro_set_threshold.argtypes = [vp, f32]
        L.tro_set_mode.argtypes = [vp, i32]
        L.tro_seq_len.argtypes = [vp, i32, C.POINTER(i32)]
        L.tro_seq_truncate.argtypes = [vp, i32, i32]
        L.tro_counters.argtypes = [vp, i32, vp]
        L.tro_seq_load_kv.argtypes = [vp, i32, i32, vp, vp]
        L.tro_seq_read_kv.argtypes = [vp, i32, i32, vp, vp]
        L.tro_forward_all.argtypes = [vp, i32, vp, vp, vp]
        L.tro_rmsnorm.argtypes = [vp, vp, i32, i32, f32, vp]; L.tro_rmsnorm.restype = None
        L.tro_rope.argtypes = [vp, i32, i32, f32]; L.tro_rope.restype = None
        L.tro_linear.argtypes = [vp, vp, i32, vp, i32, i32, vp]; L.tro_linear.restype = None
        L.tro_attend.argtypes = [vp, vp, vp, i32, i32, i32, vp]; L.tro_attend.restype = None
        L.tro_silu.argtypes = [f32]; L.tro_silu.restype = f32
        L.tro_softmax_stats.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(f32)]; L.tro_softmax_stats.restype = None
        L.tro_router_score.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32]; L.tro_router_score.restype = f32
        L.tro_linear_score.argtypes = [vp, vp, vp, i32, i32]; L.tro_linear_score.restype = f32
        L.tro_route_flag.argtypes = [f32, f32, i32, i32]; L.tro_route_flag.restype = i32
        L.tro_bf16_to_f32.argtypes = [C.c_uint16]; L.tro_bf16_to_f32.restype = f32
        L.tro_round_to_bf16.argtypes = [f32]; L.tro_round_to_bf16.restype = f32
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _check_w(a, dtype):
    want = np.float32 if dtype == F32 else np.uint16
    assert a.dtype == want and a.flags.c_contiguous, (a.dtype, want)
    return a


# ---------------------------------------------------------------- pieces

def rmsnorm(x, gain, dtype, eps):
    x = _f32(x); out = np.empty_like(x)
    lib().tro_rmsnorm(_p(x), _p(_check_w(gain, dtype)), dtype, x.size, eps, _p(out))
    return out


def rope(u, pos, theta):
    u = _f32(u).copy()
    lib().tro_rope(_p(u), u.size, int(pos), theta)
    return u


def linear(W, bias, dtype, x):
    x = _f32(x); N, K = W.shape
    assert x.size == K
    out = np.empty(N, dtype=np.float32)
    lib().tro_linear(_p(_check_w(W, dtype)), _p(None if bias is None else _check_w(bias, dtype)), dtype, _p(x), N, K, _p(out))
    return out


def attend(q, K, V):
    """q [dh], K/V [ctx][dh] -> [dh]"""
    q, K, V = _f32(q), _f32(K), _f32(V)
    ctx, dh = K.shape
    out = np.empty(dh, dtype=np.float32)
    lib().tro_attend(_p(q), _p(K), _p(V), ctx, dh, dh, _p(out))
    return out


def silu(u):
    return lib().tro_silu(float(u))


def softmax_stats(z):
    z = _f32(z)
    am, mp = C.c_int32(), C.c_float()
    lib().tro_softmax_stats(_p(z), z.size, C.byref(am), C.byref(mp))
    return am.value, mp.value


def router_score(u, w1, b1, w2, b2, dtype):
    u = _f32(u); rh, d = w1.shape
    return lib().tro_router_score(_p(u), _p(_check_w(w1, dtype)), _p(b1), _p(_check_w(w2, dtype)), _p(b2), dtype, d, rh)


def linear_score(u, w, b, dtype):
    u = np.ascontiguousarray(u, np.float32)
    return lib().tro_linear_score(_p(u), _p(_check_w(w, dtype)), _p(b), dtype, u.size)


def route_flag(score, threshold, route_dir=ROUTE_IF_BELOW, mode=JOINT):
    return lib().tro_route_flag(float(score), float(threshold), route_dir, mode)


def bf16_to_f32(bits):
    return lib().tro_bf16_to_f32(int(bits))


def round_to_bf16(f):
    return lib().tro_round_to_bf16(float(f))


# ---------------------------------------------------------------- model context

class Outputs:
    """Host output buffers of one call."""

    def __init__(self, n, d, vocab, want_logits):
        self.token = np.zeros(n, np.int32); self.conf = np.zeros(n, np.float32); self.score = np.zeros(n, np.float32)
        self.flag = np.zeros(n, np.int32); self.hidden = np.zeros((n, d), np.float32)
        self.logits = np.zeros((n, vocab), np.float32) if want_logits else None

    def struct(self):
        return Out(_p(self.token), _p(self.conf), _p(self.score), _p(self.flag), _p(self.hidden), _p(self.logits))


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: error {code}")
        self.code = code


class Model:
    """A tro context over borrowed numpy weights (dict of name -> array, per-layer names ``l{i}.wq`` ...)."""

    def __init__(self, shape: dict, weights: dict, max_batch: int, max_seq: int, route_dir=ROUTE_IF_BELOW,
                 hidden_tap=POST_FINAL_NORM, route_policy=POLICY_MLP):
        self.shape = dict(shape)
        s = self.shape
        self.cfg = Config(s["n_layers"], s["d_model"], s["n_q_heads"], s["n_kv_heads"], s["head_dim"], s["d_ffn"], s["vocab"],
                          s["rms_eps"], s["rope_theta"], s["dtype"], s["kv_dtype"], s["tie_lm_head"], s["router_hidden"],
                          s["threshold"], route_dir, hidden_tap, max_batch, max_seq, route_policy)
        self._keep = weights
        dt, L = s["dtype"], s["n_layers"]

        def one(name):
            a = weights.get(name)
            return None if a is None else _p(_check_w(a, dt))

        def per_layer(name):
            if f"l0.{name}" not in weights:
                return None
            arr = (C.c_void_p * L)(*[_p(_check_w(weights[f"l{i}.{name}"], dt)) for i in range(L)])
            self._arrs.append(arr)
            return C.cast(arr, _PP)

        self._arrs = []
        w = Weights(one("tok_emb"), one("lm_head"), one("final_norm"),
                    *[per_layer(n) for n in ("ln1", "wq", "wk", "wv", "bq", "bk", "bv", "wo", "ln2", "wg", "wu", "wd")],
                    one("r_w1"), one("r_b1"), one("r_w2"), one("r_b2"))
        self._h = C.c_void_p()
        rc = lib().tro_create(C.byref(self.cfg), C.byref(w), C.byref(self._h))
        if rc:
            raise OracleError(rc, "tro_create")

    def close(self):
        if self._h:
            lib().tro_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _out(self, n, want_logits):
        return Outputs(n, self.shape["d_model"], self.shape["vocab"], want_logits)

    def prefill(self, slots, prompts, want_logits=False):
        """prompts: list of int sequences, one per slot."""
        slots = np.ascontiguousarray(slots, dtype=np.int32)
        flat = np.ascontiguousarray(np.concatenate([np.asarray(p, dtype=np.int32) for p in prompts]), dtype=np.int32)
        offs = np.zeros(len(prompts) + 1, np.int32); offs[1:] = np.cumsum([len(p) for p in prompts])
        o = self._out(len(slots), want_logits)
        st = o.struct()
        rc = lib().tro_prefill(self._h, len(slots), _p(slots), _p(flat), _p(offs), C.byref(st))
        if rc:
            raise OracleError(rc, "tro_prefill")
        return o

    def extend(self, slots, segments, want_logits=False):
        """segments: list of int sequences, one per slot, ingested over the slot's existing cache."""
        slots = np.ascontiguousarray(slots, dtype=np.int32)
        flat = np.ascontiguousarray(np.concatenate([np.asarray(p, dtype=np.int32) for p in segments]), dtype=np.int32)
        offs = np.zeros(len(segments) + 1, np.int32); offs[1:] = np.cumsum([len(p) for p in segments])
        o = self._out(len(slots), want_logits)
        st = o.struct()
        rc = lib().tro_extend(self._h, len(slots), _p(slots), _p(flat), _p(offs), C.byref(st))
        if rc:
            raise OracleError(rc, "tro_extend")
        return o

    def decode_step(self, slots, in_tokens, want_logits=False):
        slots = np.ascontiguousarray(slots, dtype=np.int32)
        toks = np.ascontiguousarray(in_tokens, dtype=np.int32)
        o = self._out(len(slots), want_logits)
        st = o.struct()
        rc = lib().tro_decode_step(self._h, len(slots), _p(slots), _p(toks), C.byref(st))
        if rc:
            raise OracleError(rc, "tro_decode_step")
        return o

    def forward_all(self, tokens, want_logits=True):
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        hid = np.empty((t.size, self.shape["d_model"]), np.float32)
        lg = np.empty((t.size, self.shape["vocab"]), np.float32) if want_logits else None
        rc = lib().tro_forward_all(self._h, t.size, _p(t), _p(hid), _p(lg))
        if rc:
            raise OracleError(rc, "tro_forward_all")
        return hid, lg

    def seq_fork(self, src, dst):
        rc = lib().tro_seq_fork(self._h, int(src), int(dst))
        if rc:
            raise OracleError(rc, "tro_seq_fork")

    def set_threshold(self, t):
        rc = lib().tro_set_threshold(self._h, float(t))
        if rc:
            raise OracleError(rc, "tro_set_threshold")

    def set_mode(self, m):
        rc = lib().tro_set_mode(self._h, int(m))
        if rc:
            raise OracleError(rc, "tro_set_mode")

    def seq_len(self, slot):
        v = C.c_int32()
        rc = lib().tro_seq_len(self._h, int(slot), C.byref(v))
        if rc:
            raise OracleError(rc, "tro_seq_len")
        return v.value

    def seq_truncate(self, slot, new_len):
        rc = lib().tro_seq_truncate(self._h, int(slot), int(new_len))
        if rc:
            raise OracleError(rc, "tro_seq_truncate")

    def counters(self, slot):
        c = np.zeros(2, np.int64)
        rc = lib().tro_counters(self._h, int(slot), _p(c))
        if rc:
            raise OracleError(rc, "tro_counters")
        return int(c[0]), int(c[1])

    def load_kv(self, slot, k, v):
        """k, v: fp32 [layer][kv_head][len][head_dim]."""
        k, v = _f32(k), _f32(v)
        rc = lib().tro_seq_load_kv(self._h, int(slot), k.shape[2], _p(k), _p(v))
        if rc:
            raise OracleError(rc, "tro_seq_load_kv")

    def read_kv(self, slot, layer):
        n = self.seq_len(slot)
        shp = (self.shape["n_kv_heads"], n, self.shape["head_dim"])
        k = np.empty(shp, np.float32); v = np.empty(shp, np.float32)
        rc = lib().tro_seq_read_kv(self._h, int(slot), int(layer), _p(k), _p(v))
        if rc:
            raise OracleError(rc, "tro_seq_read_kv")
        return k, v
