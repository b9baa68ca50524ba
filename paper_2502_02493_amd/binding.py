"""ctypes binding of libeasyspec.so: one Python function per C entry point of
include/easyspec.h and include/easyspec_instrument.h, same names, argument marshalling only.  Nothing is computed here and there
is no fallback: if the library is missing or no GPU is usable the calls raise."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libeasyspec.so")

EASYSPEC_OK, EASYSPEC_EINVAL, EASYSPEC_ECAPACITY, EASYSPEC_ESTATE, EASYSPEC_EHIP = 0, -1, -2, -3, -4
EASYSPEC_DTYPE_F32, EASYSPEC_DTYPE_BF16 = 0, 1
EASYSPEC_POLICY_ALIGNED, EASYSPEC_POLICY_PACKED = 0, 1
EASYSPEC_MAX_BATCH, EASYSPEC_MAX_CALIB_TOKENS, EASYSPEC_MAX_SET = 16, 16, 8
EASYSPEC_MAX_TREE_WIDTH, EASYSPEC_MAX_TREE_NODES = 16, 64
EASYSPEC_MAX_CHUNKS = 64
EASYSPEC_PARALLEL_ATTENTION, EASYSPEC_PARALLEL_FULL_LAYER = 0, 1

EXPORTS = ["easyspec_create", "easyspec_destroy", "easyspec_load_weights", "easyspec_set_groups",
           "easyspec_default_groups", "easyspec_draft_step", "easyspec_calibrate", "easyspec_greedy_accept", "easyspec_greedy_accept_host",
           "easyspec_accept", "easyspec_accept_workspace_bytes", "easyspec_accept_static", "easyspec_accept_static_max_bytes", "easyspec_draft_tree_step", "easyspec_set_parallel_mode", "easyspec_stream_read", "easyspec_stream_read_sink_floats", "easyspec_attention_cut", "easyspec_weight_walk", "easyspec_attention_stage_walk",
           "easyspec_get_lens", "easyspec_truncate", "easyspec_kv_import", "easyspec_kv_export",
           "easyspec_get_hidden", "easyspec_poison_workspaces", "easyspec_step_bytes", "easyspec_profile_begin", "easyspec_profile_end",
           "easyspec_last_error"]
EASYSPEC_OP_QKV, EASYSPEC_OP_ATTN, EASYSPEC_OP_OPROJ, EASYSPEC_OP_GATEUP, EASYSPEC_OP_DOWN, EASYSPEC_OP_HEAD, EASYSPEC_OP_ALL = range(7)


class EasySpecError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"easyspec error {code}: {msg}")
        self.code = code


class easyspec_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("rms_eps", C.c_float),
                ("rope_theta", C.c_float), ("qkv_bias", C.c_int32), ("dtype", C.c_int32), ("max_batch", C.c_int32),
                ("max_ctx", C.c_int32), ("max_calib_tokens", C.c_int32)]


class easyspec_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "bq", "bk", "bv", "g_attn", "g_mlp")]


class easyspec_weights(C.Structure):
    _fields_ = [("layers", C.POINTER(easyspec_layer_weights)), ("embed", C.c_void_p), ("lm_head", C.c_void_p),
                ("g_final", C.c_void_p)]


_lib = None


def load_library():
    """Load libeasyspec.so (built by paper_2502_02493_amd.build).  Raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run `python -m paper_2502_02493_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i32 = C.c_void_p, C.c_int32
        L.easyspec_create.argtypes = [C.POINTER(easyspec_config), vp, C.POINTER(vp)]
        L.easyspec_destroy.argtypes = [vp]
        L.easyspec_destroy.restype = None
        L.easyspec_load_weights.argtypes = [vp, C.POINTER(easyspec_weights)]
        L.easyspec_set_groups.argtypes = [vp, vp, i32]
        L.easyspec_default_groups.argtypes = [i32, i32, i32, vp, C.POINTER(i32)]
        L.easyspec_draft_step.argtypes = [vp, vp, vp, vp]
        L.easyspec_set_parallel_mode.argtypes = [vp, i32]
        L.easyspec_calibrate.argtypes = [vp, vp, vp, vp, vp, i32]
        L.easyspec_draft_tree_step.argtypes = [vp, vp, vp, vp, vp, vp]
        L.easyspec_greedy_accept.argtypes = [vp, vp, i32, i32, vp, vp, vp]
        L.easyspec_greedy_accept_host.argtypes = [vp, vp, i32, i32, vp, vp]
        L.easyspec_accept.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, C.c_float, vp, vp, vp, vp]
        L.easyspec_accept_static.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, C.c_float, vp, vp, vp]
        L.easyspec_accept_static_max_bytes.argtypes = []
        L.easyspec_accept_static_max_bytes.restype = C.c_int64
        L.easyspec_accept_workspace_bytes.argtypes = [i32, i32, i32]
        L.easyspec_accept_workspace_bytes.restype = C.c_int64
        L.easyspec_get_lens.argtypes = [vp, vp, vp]
        L.easyspec_truncate.argtypes = [vp, i32, i32]
        L.easyspec_kv_import.argtypes = [vp, i32, vp, vp, i32]
        L.easyspec_kv_export.argtypes = [vp, i32, vp, vp, i32]
        L.easyspec_get_hidden.argtypes = [vp, vp, i32, C.POINTER(i32)]
        L.easyspec_step_bytes.argtypes = [vp]
        L.easyspec_poison_workspaces.argtypes = [vp]
        L.easyspec_stream_read.argtypes = [vp, C.c_int64, vp, vp]
        L.easyspec_stream_read_sink_floats.argtypes = []
        L.easyspec_attention_cut.argtypes = [C.POINTER(easyspec_config), vp, i32, i32, vp, vp]
        L.easyspec_step_bytes.restype = C.c_int64
        L.easyspec_weight_walk.argtypes = [C.POINTER(easyspec_config), i32, i32, i32, i32, vp]
        L.easyspec_attention_stage_walk.argtypes = [i32, vp]
        L.easyspec_profile_begin.argtypes = [vp, i32, i32]
        L.easyspec_profile_end.argtypes = [vp, C.POINTER(i32), C.POINTER(C.c_float), vp, vp]
        L.easyspec_last_error.argtypes = [vp]
        L.easyspec_last_error.restype = C.c_char_p
        _lib = L
    return _lib


def _ptr(x):
    """Address of a torch tensor, numpy array, raw int or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        assert x.flags["C_CONTIGUOUS"]
        return x.ctypes.data
    if hasattr(x, "data_ptr"):
        assert x.is_contiguous()
        return x.data_ptr()
    raise TypeError(type(x))


def _check(rc, ctx):
    if rc != EASYSPEC_OK:
        raise EasySpecError(rc, easyspec_last_error(ctx))


def easyspec_last_error(ctx=None) -> str:
    return load_library().easyspec_last_error(ctx).decode()


def easyspec_create(cfg: easyspec_config, hip_stream=None):
    h = C.c_void_p()
    _check(load_library().easyspec_create(C.byref(cfg), _ptr(hip_stream), C.byref(h)), None)
    return h


def easyspec_destroy(ctx):
    load_library().easyspec_destroy(ctx)


def easyspec_load_weights(ctx, weights: dict):
    """weights: the dict layout of easyspec_synth.make_weights; values are numpy arrays (host) or
    torch tensors (host or device)."""
    keep = []

    def p(a):
        if a is None:
            return None
        if isinstance(a, np.ndarray):
            a = np.ascontiguousarray(a)
        keep.append(a)
        return _ptr(a)

    n = len(weights["layers"])
    arr = (easyspec_layer_weights * n)()
    for i, lw in enumerate(weights["layers"]):
        for name in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g_attn", "g_mlp"):
            setattr(arr[i], name, p(lw[name]))
        for name in ("bq", "bk", "bv"):
            setattr(arr[i], name, p(lw.get(name)))
    w = easyspec_weights(arr, p(weights["embed"]), p(weights["lm_head"]), p(weights["g_final"]))
    _check(load_library().easyspec_load_weights(ctx, C.byref(w)), ctx)


def easyspec_set_groups(ctx, bounds):
    b = np.ascontiguousarray(bounds, dtype=np.int32)
    _check(load_library().easyspec_set_groups(ctx, _ptr(b), b.size - 1), ctx)


def easyspec_default_groups(n_layers: int, N: int, policy: int) -> np.ndarray:
    b = np.zeros(max(n_layers, 0) + 2, dtype=np.int32)
    n = C.c_int32(0)
    _check(load_library().easyspec_default_groups(n_layers, N, policy, _ptr(b), C.byref(n)), None)
    return b[: n.value + 1].copy()


def easyspec_draft_step(ctx, tokens_in, tokens_out, logits_out=None):
    _check(load_library().easyspec_draft_step(ctx, _ptr(tokens_in), _ptr(tokens_out), _ptr(logits_out)), ctx)


def easyspec_calibrate(ctx, tokens, n_tokens, next_token_out, logits_out=None, logits_rows=0):
    n = np.ascontiguousarray(n_tokens, dtype=np.int32)
    _check(load_library().easyspec_calibrate(ctx, _ptr(tokens), _ptr(n), _ptr(next_token_out), _ptr(logits_out),
                                             int(logits_rows)), ctx)


def easyspec_set_parallel_mode(ctx, mode: int):
    _check(load_library().easyspec_set_parallel_mode(ctx, int(mode)), ctx)


def easyspec_draft_tree_step(ctx, tokens_in, n_nodes, parents, tokens_out, logits_out=None):
    n = np.ascontiguousarray(n_nodes, dtype=np.int32)
    p = np.ascontiguousarray(parents, dtype=np.int32)
    assert p.size == n.size * EASYSPEC_MAX_TREE_WIDTH
    _check(load_library().easyspec_draft_tree_step(ctx, _ptr(tokens_in), _ptr(n), _ptr(p), _ptr(tokens_out), _ptr(logits_out)), ctx)


def easyspec_greedy_accept(draft, target_argmax, batch, gamma, accept_len, bonus, hip_stream=None):
    _check(load_library().easyspec_greedy_accept(_ptr(draft), _ptr(target_argmax), batch, gamma, _ptr(accept_len),
                                                 _ptr(bonus), _ptr(hip_stream)), None)


def easyspec_greedy_accept_host(draft, target_argmax, batch, gamma, accept_len, bonus):
    _check(load_library().easyspec_greedy_accept_host(_ptr(draft), _ptr(target_argmax), batch, gamma, _ptr(accept_len),
                                                      _ptr(bonus)), None)


def easyspec_accept(draft, draft_logits, target_logits, r, u, batch, gamma, vocab, temperature, accept_len, bonus,
                    workspace, hip_stream=None):
    _check(load_library().easyspec_accept(_ptr(draft), _ptr(draft_logits), _ptr(target_logits), _ptr(r), _ptr(u), batch,
                                          gamma, vocab, float(temperature), _ptr(accept_len), _ptr(bonus), _ptr(workspace),
                                          _ptr(hip_stream)), None)


def easyspec_accept_static(draft, draft_logits, target_logits, r, u, batch, gamma, vocab, temperature, accept_len, bonus,
                           hip_stream=None):
    _check(load_library().easyspec_accept_static(_ptr(draft), _ptr(draft_logits), _ptr(target_logits), _ptr(r), _ptr(u), batch,
                                                 gamma, vocab, float(temperature), _ptr(accept_len), _ptr(bonus),
                                                 _ptr(hip_stream)), None)


def easyspec_accept_static_max_bytes() -> int:
    return int(load_library().easyspec_accept_static_max_bytes())


def easyspec_accept_workspace_bytes(batch: int, gamma: int, vocab: int) -> int:
    return int(load_library().easyspec_accept_workspace_bytes(batch, gamma, vocab))


def easyspec_stream_read(buf, nbytes: int, sink, hip_stream=None):
    _check(load_library().easyspec_stream_read(_ptr(buf), int(nbytes), _ptr(sink), _ptr(hip_stream)), None)


def easyspec_stream_read_sink_floats() -> int:
    return int(load_library().easyspec_stream_read_sink_floats())


def easyspec_attention_cut(cfg: easyspec_config, ctx_lens, n_layers_in_set: int, with_ranges=True):
    """(waves per workgroup, n_chunks[n_cols], ranges[n_cols][EASYSPEC_MAX_CHUNKS][8][2] or None)."""
    lens = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    n_chunks = np.zeros(len(lens), np.int32)
    ranges = np.zeros((len(lens), EASYSPEC_MAX_CHUNKS, 8, 2), np.int32) if with_ranges else None
    rc = load_library().easyspec_attention_cut(C.byref(cfg), _ptr(lens), len(lens), int(n_layers_in_set), _ptr(n_chunks),
                                               _ptr(ranges))
    if rc < 0:
        _check(rc, None)
    return rc, n_chunks, ranges


EASYSPEC_WALK_FIELDS = 16
WALK_NAMES = ("grid", "waves", "units_per_wg", "tile_rows", "fragments", "w_max", "w_pieces", "w_out_of_range", "x_max",
              "x_slot_elems", "x_out_of_range", "tiles", "missed_tiles", "repeated_tiles", "reread_tiles", "uncovered_pieces")


def easyspec_weight_walk(cfg: easyspec_config, op: int, n_cols: int, n_layers_in_set: int, full_layer: bool = False) -> dict:
    rep = np.zeros(EASYSPEC_WALK_FIELDS, np.int64)
    _check(load_library().easyspec_weight_walk(C.byref(cfg), int(op), int(n_cols), int(n_layers_in_set), int(bool(full_layer)),
                                               _ptr(rep)), None)
    return dict(zip(WALK_NAMES, (int(v) for v in rep)))


EASYSPEC_STAGE_FIELDS = 9
STAGE_NAMES = ("stored", "distinct_places", "highest_place", "places", "fetched", "wrong_piece", "unused_rows", "misplaced_scores",
               "bank_conflicts")


def easyspec_attention_stage_walk(n_loads: int) -> dict:
    rep = np.zeros(EASYSPEC_STAGE_FIELDS, np.int64)
    _check(load_library().easyspec_attention_stage_walk(int(n_loads), _ptr(rep)), None)
    return dict(zip(STAGE_NAMES, (int(v) for v in rep)))


def easyspec_get_lens(ctx, max_batch: int):
    p, f = np.zeros(max_batch, np.int32), np.zeros(max_batch, np.int32)
    _check(load_library().easyspec_get_lens(ctx, _ptr(p), _ptr(f)), ctx)
    return p, f


def easyspec_truncate(ctx, b: int, new_precise_len: int):
    _check(load_library().easyspec_truncate(ctx, b, new_precise_len), ctx)


def easyspec_kv_import(ctx, b: int, k, v, n_slots: int):
    _check(load_library().easyspec_kv_import(ctx, b, _ptr(k), _ptr(v), n_slots), ctx)


def easyspec_kv_export(ctx, b: int, k, v, n_slots: int):
    _check(load_library().easyspec_kv_export(ctx, b, _ptr(k), _ptr(v), n_slots), ctx)


def easyspec_get_hidden(ctx, out, max_rows: int) -> int:
    n = C.c_int32(0)
    _check(load_library().easyspec_get_hidden(ctx, _ptr(out), max_rows, C.byref(n)), ctx)
    return n.value


def easyspec_poison_workspaces(ctx):
    _check(load_library().easyspec_poison_workspaces(ctx), ctx)


def easyspec_step_bytes(ctx) -> int:
    return int(load_library().easyspec_step_bytes(ctx))


def easyspec_profile_begin(ctx, op: int, max_launches: int):
    _check(load_library().easyspec_profile_begin(ctx, op, max_launches), ctx)


def easyspec_profile_end(ctx, per_launch=None, per_launch_op=None):
    """Returns (timed launches, total milliseconds); per_launch / per_launch_op: float32 / int32 numpy arrays of
    at least max_launches entries that receive each launch's milliseconds and kernel class."""
    n, ms = C.c_int32(0), C.c_float(0.0)
    assert per_launch is None or per_launch.dtype == np.float32
    assert per_launch_op is None or per_launch_op.dtype == np.int32
    _check(load_library().easyspec_profile_end(ctx, C.byref(n), C.byref(ms), _ptr(per_launch), _ptr(per_launch_op)), ctx)
    return n.value, ms.value


def make_config(shape: dict, max_batch: int, max_ctx: int, max_calib_tokens: int) -> easyspec_config:
    """easyspec_config from a model-shape dict (fields of easyspec_synth.model_shape)."""
    return easyspec_config(shape["n_layers"], shape["d_model"], shape["n_q_heads"], shape["n_kv_heads"],
                           shape["head_dim"], shape["d_ffn"], shape["vocab"], shape["rms_eps"], shape["rope_theta"],
                           int(shape["qkv_bias"]), EASYSPEC_DTYPE_BF16 if shape["dtype"] == "bf16" else EASYSPEC_DTYPE_F32,
                           max_batch, max_ctx, max_calib_tokens)
