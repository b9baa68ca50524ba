"""ctypes front end of the EasySpec CPU oracle (oracle/easyspec_oracle.c).

TEST INFRASTRUCTURE ONLY.  Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline
leg may import this module.  It builds the C file with gcc on first use and holds no
arithmetic of its own beyond the greedy speculative-decoding loop harness at the bottom,
which only sequences oracle calls (paper Alg. 3 at temperature 0, Sec. 3.2 iteration order).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "easyspec_oracle.c")
_LIB = os.path.join(_HERE, "libeasyspec_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over output rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim",
                                         "d_ffn", "vocab", "qkv_bias", "bf16", "max_ctx")] + \
               [("rms_eps", C.c_double), ("rope_theta", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        # EASYSPEC_ORACLE_LIB: another build of the same source (the sanitizer build of tests/test_oracle_sanitized.py)
        L = C.CDLL(os.environ.get("EASYSPEC_ORACLE_LIB") or build())
        vp, i32, dp, fp, ip = C.c_void_p, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_float), C.POINTER(C.c_int32)
        L.eso_bf16_round.restype = C.c_double
        L.eso_bf16_round.argtypes = [C.c_double]
        L.eso_bf16_pair_round.restype = C.c_double
        L.eso_bf16_pair_round.argtypes = [C.c_double]
        L.eso_model_set_rounding.restype = C.c_int
        L.eso_model_set_rounding.argtypes = [vp, i32, i32]
        L.eso_matvec.argtypes = [vp, C.c_int, vp, C.c_double, C.c_int, C.c_int, dp, dp]
        L.eso_rmsnorm.argtypes = [dp, fp, C.c_int, C.c_double, dp]
        L.eso_rope.argtypes = [dp, C.c_int, C.c_int, C.c_double]
        L.eso_silu.restype = C.c_double
        L.eso_silu.argtypes = [C.c_double]
        L.eso_softmax.argtypes = [dp, C.c_int]
        L.eso_argmax.restype = i32
        L.eso_argmax.argtypes = [dp, C.c_int, dp]
        L.eso_model_create.restype = vp
        L.eso_model_create.argtypes = [C.POINTER(_Config)]
        L.eso_model_set_layer.argtypes = [vp, C.c_int] + [vp] * 12
        L.eso_model_set_top.argtypes = [vp, vp, vp, vp]
        L.eso_model_destroy.argtypes = [vp]
        L.eso_seq_create.restype = vp
        L.eso_seq_create.argtypes = [vp]
        L.eso_seq_destroy.argtypes = [vp]
        L.eso_seq_k.restype = fp
        L.eso_seq_k.argtypes = [vp]
        L.eso_seq_v.restype = fp
        L.eso_seq_v.argtypes = [vp]
        L.eso_seq_precise.restype = i32
        L.eso_seq_precise.argtypes = [vp]
        L.eso_seq_fuzzy.restype = i32
        L.eso_seq_fuzzy.argtypes = [vp]
        L.eso_seq_set_lens.argtypes = [vp, i32, i32]
        L.eso_seq_set_full_layer.argtypes = [vp, i32]
        L.eso_seq_enable_attn_tap.restype = dp
        L.eso_seq_enable_attn_tap.argtypes = [vp]
        L.eso_sequential_step.argtypes = [vp, i32, dp, dp]
        L.eso_fuzzy_step.argtypes = [vp, ip, i32, i32, dp, dp]
        L.eso_fuzzy_tree_step.argtypes = [vp, ip, i32, i32, ip, ip, dp, dp]
        L.eso_calibrate.argtypes = [vp, ip, i32, dp, dp]
        L.eso_calibrate_last.argtypes = [vp, ip, i32, dp]
        L.eso_greedy_accept.argtypes = [ip, ip, i32, ip, ip]
        L.eso_default_groups.argtypes = [i32, i32, i32, ip, ip]
        fp = C.POINTER(C.c_float)
        L.eso_accept.argtypes = [ip, fp, fp, fp, C.c_float, i32, i32, C.c_double, ip, ip, dp]
        _lib = L
    return _lib


def _dp(a):
    return a.ctypes.data_as(C.POINTER(C.c_double)) if a is not None else None


def _ip(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _vp(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


# ------------------------------------------------------------------------------ primitives

def bf16_round(x: float) -> float:
    return lib().eso_bf16_round(float(x))


def bf16_pair_round(x: float) -> float:
    """x carried as two bf16 terms: bf16(x) + bf16(x - bf16(x))."""
    return lib().eso_bf16_pair_round(float(x))


ACT_PLAIN, ACT_SINGLE, ACT_PAIR = 0, 1, 2     # ESO_ACT_* of the C file


def matvec(w: np.ndarray, x: np.ndarray, bias: np.ndarray | None = None, scale: float = 1.0) -> np.ndarray:
    """scale * (w @ x) + bias;  w: [rows, cols] float32 or uint16 (bf16 bits)."""
    w = np.ascontiguousarray(w)
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.empty(w.shape[0], dtype=np.float64)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    lib().eso_matvec(_vp(w), int(w.dtype == np.uint16), _vp(b), float(scale), w.shape[0], w.shape[1], _dp(x), _dp(y))
    return y


def rmsnorm(x, g, eps):
    x = np.ascontiguousarray(x, dtype=np.float64)
    g = np.ascontiguousarray(g, dtype=np.float32)
    y = np.empty_like(x)
    lib().eso_rmsnorm(_dp(x), g.ctypes.data_as(C.POINTER(C.c_float)), x.size, float(eps), _dp(y))
    return y


def rope(x, pos, theta):
    y = np.array(x, dtype=np.float64, copy=True)
    lib().eso_rope(_dp(y), y.size, int(pos), float(theta))
    return y


def silu(z: float) -> float:
    return lib().eso_silu(float(z))


def softmax(s):
    y = np.array(s, dtype=np.float64, copy=True)
    lib().eso_softmax(_dp(y), y.size)
    return y


def argmax(x, with_margin: bool = False):
    x = np.ascontiguousarray(x, dtype=np.float64)
    m = C.c_double(0.0)
    i = lib().eso_argmax(_dp(x), x.size, C.byref(m) if with_margin else None)
    return (int(i), float(m.value)) if with_margin else int(i)


def greedy_accept(draft, target):
    draft = np.ascontiguousarray(draft, dtype=np.int32)
    target = np.ascontiguousarray(target, dtype=np.int32)
    assert target.size == draft.size + 1
    m, b = C.c_int32(-1), C.c_int32(-1)
    lib().eso_greedy_accept(_ip(draft), _ip(target), draft.size, C.byref(m), C.byref(b))
    return int(m.value), int(b.value)


def accept(draft, draft_logits, target_logits, r, u, temperature, with_margin: bool = False):
    """Acceptance by speculative sampling (paper Alg. 3 / Sec. 2.1) for one sequence; r [gamma] and
    u are the uniform random numbers.  Returns (accept_len, bonus[, margin])."""
    draft = np.ascontiguousarray(draft, dtype=np.int32)
    dl = np.ascontiguousarray(draft_logits, dtype=np.float32)
    tl = np.ascontiguousarray(target_logits, dtype=np.float32)
    r = np.ascontiguousarray(r, dtype=np.float32)
    gamma = draft.size
    V = tl.shape[-1]
    assert tl.shape == (gamma + 1, V) and dl.shape == (gamma, V) and r.size == gamma
    fp = C.POINTER(C.c_float)
    m, b, mg = C.c_int32(-1), C.c_int32(-1), C.c_double(0.0)
    rc = lib().eso_accept(_ip(draft), dl.ctypes.data_as(fp), tl.ctypes.data_as(fp), r.ctypes.data_as(fp), float(np.float32(u)),
                          gamma, V, float(temperature), C.byref(m), C.byref(b), C.byref(mg))
    if rc != 0:
        raise ValueError("bad accept arguments")
    return (int(m.value), int(b.value), float(mg.value)) if with_margin else (int(m.value), int(b.value))


def default_groups(n_layers: int, group_size: int, policy: str = "aligned"):
    """Set boundaries [0, ..., L] of the layer-parallel strategy (paper Sec. 3.1.1)."""
    b = np.zeros(n_layers + 1, dtype=np.int32)
    n = C.c_int32(0)
    rc = lib().eso_default_groups(n_layers, group_size, {"aligned": 0, "packed": 1}[policy], _ip(b), C.byref(n))
    if rc != 0:
        raise ValueError("bad strategy arguments")
    return b[: n.value + 1].copy()


# ------------------------------------------------------------------------------ model / sequence

class Model:
    """Holds references to the caller's parameter arrays (no copies are made)."""

    def __init__(self, cfg: dict, weights: dict, max_ctx: int):
        self.cfg = dict(cfg)
        self.max_ctx = int(max_ctx)
        self.bf16 = cfg["dtype"] == "bf16"
        c = _Config(cfg["n_layers"], cfg["d_model"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"],
                    cfg["d_ffn"], cfg["vocab"], int(cfg["qkv_bias"]), int(self.bf16), self.max_ctx,
                    float(cfg["rms_eps"]), float(cfg["rope_theta"]))
        self._h = lib().eso_model_create(C.byref(c))
        if not self._h:
            raise ValueError("bad oracle config")
        self._keep = []
        mat_dt = np.uint16 if self.bf16 else np.float32

        def mat(a, shape):
            a = np.ascontiguousarray(a)
            assert a.dtype == mat_dt and a.shape == tuple(shape), (a.dtype, a.shape, shape)
            self._keep.append(a)
            return _vp(a)

        def vec(a, n):
            if a is None:
                return None
            a = np.ascontiguousarray(a, dtype=np.float32)
            assert a.shape == (n,)
            self._keep.append(a)
            return _vp(a)

        d, hq, hkv, hd, f, v = (cfg["d_model"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"],
                                cfg["d_ffn"], cfg["vocab"])
        for i, lw in enumerate(weights["layers"]):
            lib().eso_model_set_layer(
                self._h, i, mat(lw["wq"], (hq * hd, d)), mat(lw["wk"], (hkv * hd, d)), mat(lw["wv"], (hkv * hd, d)),
                mat(lw["wo"], (d, hq * hd)), mat(lw["wg"], (f, d)), mat(lw["wu"], (f, d)), mat(lw["wd"], (d, f)),
                vec(lw.get("bq"), hq * hd), vec(lw.get("bk"), hkv * hd), vec(lw.get("bv"), hkv * hd),
                vec(lw["g_attn"], d), vec(lw["g_mlp"], d))
        lib().eso_model_set_top(self._h, mat(weights["embed"], (v, d)), vec(weights["g_final"], d),
                                mat(weights["lm_head"], (v, d)))

    def set_rounding(self, act_mode: int, kv_bf16: bool):
        """Where the model rounds: act_mode ACT_PLAIN (activations unrounded, RMSNorm as written: the plain
        reference), ACT_SINGLE (one bf16 number) or ACT_PAIR (two bf16 terms, RMSNorm carried in two parts:
        the HIP library's operand format); kv_bf16: cache entries rounded to bf16."""
        if lib().eso_model_set_rounding(self._h, int(act_mode), int(bool(kv_bf16))) != 0:
            raise ValueError("bad rounding mode")
        return self

    def __del__(self):
        if getattr(self, "_h", None):
            lib().eso_model_destroy(self._h)
            self._h = None


class Sequence:
    """One sequence's draft KV cache with its precise / fuzzy lengths."""

    def __init__(self, model: Model):
        self.model = model
        self._h = lib().eso_seq_create(model._h)
        c = model.cfg
        shape = (c["n_layers"], c["n_kv_heads"], model.max_ctx, c["head_dim"])
        n = int(np.prod(shape))
        self.K = np.ctypeslib.as_array(lib().eso_seq_k(self._h), shape=(n,)).reshape(shape)
        self.V = np.ctypeslib.as_array(lib().eso_seq_v(self._h), shape=(n,)).reshape(shape)
        self._tap = None

    def __del__(self):
        if getattr(self, "_h", None):
            self.K = self.V = None
            lib().eso_seq_destroy(self._h)
            self._h = None

    @property
    def precise(self):
        return lib().eso_seq_precise(self._h)

    @property
    def fuzzy(self):
        return lib().eso_seq_fuzzy(self._h)

    def set_lens(self, precise, fuzzy=0):
        lib().eso_seq_set_lens(self._h, int(precise), int(fuzzy))

    def import_kv(self, k, v):
        """k, v: [L, Hkv, n, hd] float32 or bf16 bits; becomes the precise prefix."""
        if k.dtype == np.uint16:
            k = (k.astype(np.uint32) << np.uint32(16)).view(np.float32)
            v = (v.astype(np.uint32) << np.uint32(16)).view(np.float32)
        n = k.shape[2]
        self.K[:, :, :n, :] = k
        self.V[:, :, :n, :] = v
        self.set_lens(n, 0)

    def set_full_layer(self, on: bool):
        """Fuzzy steps run every layer of a set, attention and MLP, from the set's input (the
        full-layer ablation of paper App. B) instead of Alg. 2."""
        self.full_layer = bool(on)
        lib().eso_seq_set_full_layer(self._h, int(self.full_layer))

    def clone(self):
        s = Sequence(self.model)
        s.K[...] = self.K
        s.V[...] = self.V
        s.set_lens(self.precise, self.fuzzy)
        s.set_full_layer(getattr(self, "full_layer", False))
        return s

    def attn_tap(self):
        """Enable and return the [L, d] array of Attnoutput_i of the last single-token step."""
        if self._tap is None:
            c = self.model.cfg
            p = lib().eso_seq_enable_attn_tap(self._h)
            self._tap = np.ctypeslib.as_array(p, shape=(c["n_layers"] * c["d_model"],)).reshape(
                c["n_layers"], c["d_model"])
        return self._tap

    def sequential_step(self, token, want_hidden=False):
        c = self.model.cfg
        logits = np.empty(c["vocab"], dtype=np.float64)
        hid = np.empty(c["d_model"], dtype=np.float64) if want_hidden else None
        if lib().eso_sequential_step(self._h, int(token), _dp(logits), _dp(hid)) != 0:
            raise RuntimeError("oracle sequential_step: bad state or arguments")
        return (logits, hid) if want_hidden else logits

    def fuzzy_step(self, bounds, token, want_hidden=False):
        c = self.model.cfg
        b = np.ascontiguousarray(bounds, dtype=np.int32)
        logits = np.empty(c["vocab"], dtype=np.float64)
        hid = np.empty(c["d_model"], dtype=np.float64) if want_hidden else None
        if lib().eso_fuzzy_step(self._h, _ip(b), b.size - 1, int(token), _dp(logits), _dp(hid)) != 0:
            raise RuntimeError("oracle fuzzy_step: bad state or arguments")
        return (logits, hid) if want_hidden else logits

    def fuzzy_tree_step(self, bounds, tokens, parents, want_hidden=False):
        """One level of a token tree (paper App. C): node j is the child of tree node parents[j]
        (-1: of the last precise token).  Returns logits [n, V]."""
        c = self.model.cfg
        b = np.ascontiguousarray(bounds, dtype=np.int32)
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        p = np.ascontiguousarray(parents, dtype=np.int32)
        assert t.size == p.size
        logits = np.empty((t.size, c["vocab"]), dtype=np.float64)
        hid = np.empty((t.size, c["d_model"]), dtype=np.float64) if want_hidden else None
        if lib().eso_fuzzy_tree_step(self._h, _ip(b), b.size - 1, t.size, _ip(t), _ip(p), _dp(logits), _dp(hid)) != 0:
            raise RuntimeError("oracle fuzzy_tree_step: bad state or arguments")
        return (logits, hid) if want_hidden else logits

    def calibrate(self, tokens, all_rows=True, want_hidden=False):
        """Returns logits [n, V] (all_rows) or [V] (last row only)."""
        c = self.model.cfg
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        n = t.size
        if all_rows:
            logits = np.empty((n, c["vocab"]), dtype=np.float64)
            hid = np.empty((n, c["d_model"]), dtype=np.float64) if want_hidden else None
            rc = lib().eso_calibrate(self._h, _ip(t), n, _dp(logits), _dp(hid))
        else:
            assert not want_hidden
            logits = np.empty(c["vocab"], dtype=np.float64)
            hid = None
            rc = lib().eso_calibrate_last(self._h, _ip(t), n, _dp(logits))
        if rc != 0:
            raise RuntimeError("oracle calibrate: bad state or arguments")
        return (logits, hid) if want_hidden else logits


# ------------------------------------------------------------------------------ loop harness

def vanilla_greedy(base: Sequence, prompt, n_new: int):
    """Greedy decoding of the base model alone: the reference output of lossless decoding."""
    logits = base.calibrate(prompt, all_rows=False)
    out = []
    for _ in range(n_new):
        tok = argmax(logits)
        out.append(tok)
        logits = base.sequential_step(tok)
    return out


def speculative_greedy(draft: Sequence, base: Sequence, prompt, bounds, gamma: int, n_new: int):
    """Three-stage iterations (paper Fig. 1 / Sec. 3.2): calibration gives the first draft
    token, gamma-1 fuzzy steps give the rest, the base model verifies all gamma in one
    forward, greedy acceptance keeps m of them plus the bonus token; the next calibration
    re-inputs the accepted tokens and the bonus token.  Returns (tokens, accept_lengths)."""
    prompt = [int(t) for t in prompt]
    out, accepts = [], []
    # the first iteration's "calibration" is the prompt prefill; the base model has consumed
    # everything but the last known token, which it receives together with the drafted ones
    calib_tokens = list(prompt)
    base.calibrate(prompt[:-1], all_rows=False) if len(prompt) > 1 else None
    last = prompt[-1]
    while len(out) < n_new:
        d_logits = draft.calibrate(calib_tokens, all_rows=False)
        drafted = [argmax(d_logits)]
        for _ in range(gamma - 1):
            drafted.append(argmax(draft.fuzzy_step(bounds, drafted[-1])))
        p0 = base.precise
        v_logits = base.calibrate([last] + drafted, all_rows=True)       # p_1 .. p_{gamma+1}
        target = [argmax(v_logits[r]) for r in range(gamma + 1)]
        m, bonus = greedy_accept(drafted, target)
        base.set_lens(p0 + 1 + m, 0)                                      # keep `last` + accepted tokens
        accepts.append(m)
        out.extend(drafted[:m] + [bonus])
        calib_tokens = drafted[:m] + [bonus]
        last = bonus
    return out[:n_new], accepts
