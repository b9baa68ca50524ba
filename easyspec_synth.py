"""Seeded synthetic inputs for the EasySpec draft hot path.

This module only *draws* inputs: model shapes, random-init parameters, token ids and
synthetic KV prefixes.  It contains none of the method's arithmetic (no norm, no
attention, no projection) and is the one piece of code that both the CPU oracle's tests
and the HIP path's tests / bench may import, so that both sides see identical bits.

Every tensor is drawn from its own counter-based Philox stream keyed by
(seed, tensor id, row chunk), which makes generation order-free, thread-safe and
identical on every machine and thread count.

Parameter recipe (the paper evaluates trained checkpoints that are not available here; the
benchmark configuration asks for random-init weights of the same shapes):
  * projection matrices, embedding, LM head, QKV biases ~ N(0, 0.02^2)
  * RMSNorm gains ~ 1 + N(0, 0.02^2)   (a gain drawn around 0 would null every block)
  * LM head is untied from the embedding
  * for bf16 models every parameter is rounded to bf16 (round-to-nearest-even); matrices
    are handed out as uint16 bit patterns, vectors as float32 holding bf16-exact values.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

# --------------------------------------------------------------------------------------
# model shapes
# --------------------------------------------------------------------------------------

_SHAPES = {
    # Tiny fp32 Llama-style decoder (CPU-seconds scale).
    "tiny": dict(n_layers=4, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ffn=1024,
                 vocab=1024, rms_eps=1e-6, rope_theta=10000.0, qkv_bias=0, dtype="fp32"),
    # Tiny Qwen2-style (7 query heads per KV head, QKV bias) for odd-shape coverage.
    "tiny_qwen": dict(n_layers=5, d_model=448, n_q_heads=7, n_kv_heads=1, head_dim=64, d_ffn=1184,
                      vocab=1000, rms_eps=1e-6, rope_theta=1000000.0, qkv_bias=1, dtype="fp32"),
    # Llama-3-8B shape.
    "llama3_8b": dict(n_layers=32, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128,
                      d_ffn=14336, vocab=128256, rms_eps=1e-5, rope_theta=500000.0, qkv_bias=0,
                      dtype="bf16"),
    # Qwen2-7B shape.
    "qwen2_7b": dict(n_layers=28, d_model=3584, n_q_heads=28, n_kv_heads=4, head_dim=128,
                     d_ffn=18944, vocab=152064, rms_eps=1e-6, rope_theta=1000000.0, qkv_bias=1,
                     dtype="bf16"),
}


def model_shape(name: str, **overrides) -> dict:
    """Return a copy of a named model shape; keyword overrides replace fields
    (e.g. ``model_shape("llama3_8b", n_layers=6, vocab=8192)`` for a reduced-depth case)."""
    cfg = dict(_SHAPES[name])
    cfg.update(overrides)
    cfg["name"] = name
    return cfg


# --------------------------------------------------------------------------------------
# bf16 storage format helpers (format conversion only)
# --------------------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even.  Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u >> np.uint32(16)
    r &= np.uint32(1)
    r += np.uint32(0x7FFF)
    r += u
    r >>= np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------------------
# seeded draws
# --------------------------------------------------------------------------------------

_CHUNK_ELEMS = 1 << 22


def _n_workers() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def _normal_rows(seed: int, tensor_id: int, chunk: int, shape) -> np.ndarray:
    g = np.random.Generator(np.random.Philox(key=[int(seed) & (2**64 - 1), (tensor_id << 20) + chunk]))
    return g.standard_normal(shape, dtype=np.float32)


def _draw_matrix(seed, tensor_id, rows, cols, std, mean, dtype, pool):
    """N(mean, std^2) matrix [rows, cols]; float32 or bf16 bits."""
    out = np.empty((rows, cols), dtype=np.uint16 if dtype == "bf16" else np.float32)
    step = max(1, _CHUNK_ELEMS // cols)

    def work(ci):
        r0 = ci * step
        r1 = min(rows, r0 + step)
        blk = _normal_rows(seed, tensor_id, ci, (r1 - r0, cols))
        blk *= np.float32(std)
        if mean != 0.0:
            blk += np.float32(mean)
        out[r0:r1] = f32_to_bf16_bits(blk) if dtype == "bf16" else blk

    n_chunks = (rows + step - 1) // step
    if pool is None or n_chunks == 1:
        for ci in range(n_chunks):
            work(ci)
    else:
        list(pool.map(work, range(n_chunks)))
    return out


def _draw_vector(seed, tensor_id, n, std, mean, dtype):
    v = _normal_rows(seed, tensor_id, 0, (n,)) * np.float32(std) + np.float32(mean)
    if dtype == "bf16":
        v = bf16_bits_to_f32(f32_to_bf16_bits(v))
    return v.astype(np.float32)


# tensor ids: layer l uses ids 16*l + k ; top-level tensors use ids from 1<<16
_K = dict(wq=0, wk=1, wv=2, wo=3, wg=4, wu=5, wd=6, bq=7, bk=8, bv=9, g_attn=10, g_mlp=11)
_TOP = dict(embed=(1 << 16), lm_head=(1 << 16) + 1, g_final=(1 << 16) + 2)


def make_weights(cfg: dict, seed: int, std: float = 0.02) -> dict:
    """Random-init parameters of a decoder with shape ``cfg``.

    Returns ``{"layers": [ {wq, wk, wv, wo, wg, wu, wd, g_attn, g_mlp[, bq, bk, bv]} ... ],
    "embed", "lm_head", "g_final"}``.  Matrices are row-major ``[out, in]`` numpy arrays
    (float32, or uint16 bf16 bits when ``cfg["dtype"] == "bf16"``); vectors are float32.
    """
    d, hq, hkv, hd, f, v = (cfg["d_model"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"],
                            cfg["d_ffn"], cfg["vocab"])
    dt = cfg["dtype"]
    pool = ThreadPoolExecutor(_n_workers()) if max(d * f, v * d) > _CHUNK_ELEMS else None
    try:
        layers = []
        for l in range(cfg["n_layers"]):
            t = 16 * l
            lw = dict(
                wq=_draw_matrix(seed, t + _K["wq"], hq * hd, d, std, 0.0, dt, pool),
                wk=_draw_matrix(seed, t + _K["wk"], hkv * hd, d, std, 0.0, dt, pool),
                wv=_draw_matrix(seed, t + _K["wv"], hkv * hd, d, std, 0.0, dt, pool),
                wo=_draw_matrix(seed, t + _K["wo"], d, hq * hd, std, 0.0, dt, pool),
                wg=_draw_matrix(seed, t + _K["wg"], f, d, std, 0.0, dt, pool),
                wu=_draw_matrix(seed, t + _K["wu"], f, d, std, 0.0, dt, pool),
                wd=_draw_matrix(seed, t + _K["wd"], d, f, std, 0.0, dt, pool),
                g_attn=_draw_vector(seed, t + _K["g_attn"], d, std, 1.0, dt),
                g_mlp=_draw_vector(seed, t + _K["g_mlp"], d, std, 1.0, dt),
            )
            if cfg["qkv_bias"]:
                lw["bq"] = _draw_vector(seed, t + _K["bq"], hq * hd, std, 0.0, dt)
                lw["bk"] = _draw_vector(seed, t + _K["bk"], hkv * hd, std, 0.0, dt)
                lw["bv"] = _draw_vector(seed, t + _K["bv"], hkv * hd, std, 0.0, dt)
            layers.append(lw)
        return dict(
            layers=layers,
            embed=_draw_matrix(seed, _TOP["embed"], v, d, std, 0.0, dt, pool),
            lm_head=_draw_matrix(seed, _TOP["lm_head"], v, d, std, 0.0, dt, pool),
            g_final=_draw_vector(seed, _TOP["g_final"], d, std, 1.0, dt),
        )
    finally:
        if pool is not None:
            pool.shutdown()


def make_tokens(seed: int, n: int, vocab: int) -> np.ndarray:
    """``n`` token ids uniform in [0, vocab), int32."""
    g = np.random.Generator(np.random.Philox(key=[int(seed) & (2**64 - 1), (1 << 40) + 7]))
    return g.integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


def make_accept_lengths(seed: int, n_iters: int, gamma: int) -> np.ndarray:
    """Per-iteration acceptance lengths uniform in 0..gamma (calibration-dominant workload)."""
    g = np.random.Generator(np.random.Philox(key=[int(seed) & (2**64 - 1), (1 << 40) + 11]))
    return g.integers(0, gamma + 1, size=n_iters, dtype=np.int64).astype(np.int32)


def make_uniforms(seed: int, n: int) -> np.ndarray:
    """n float32 uniforms in [0, 1): the random numbers speculative sampling draws, handed to
    both implementations as inputs."""
    g = np.random.Generator(np.random.Philox(key=[int(seed) & (2**64 - 1), (1 << 40) + 13]))
    return g.random(n, dtype=np.float32)


def make_logits(seed: int, rows: int, vocab: int, std: float = 2.0) -> np.ndarray:
    """[rows, vocab] float32 N(0, std) logits for acceptance tests (std 2 gives softmax
    distributions with a few dominant tokens, as a trained model's are)."""
    g = np.random.Generator(np.random.Philox(key=[int(seed) & (2**64 - 1), (1 << 40) + 17]))
    return (g.standard_normal((rows, vocab), dtype=np.float32) * np.float32(std)).astype(np.float32)


def make_kv_prefix(cfg: dict, seed: int, n_slots: int, seq: int = 0):
    """Synthetic KV prefix standing in for a prefilled context: two arrays
    ``[n_layers, n_kv_heads, n_slots, head_dim]`` of N(0,1) values in the model's storage
    dtype (float32, or uint16 bf16 bits).  The same buffers are imported by both sides."""
    L, hkv, hd = cfg["n_layers"], cfg["n_kv_heads"], cfg["head_dim"]
    dt = cfg["dtype"]
    pool = ThreadPoolExecutor(_n_workers()) if L * hkv * n_slots * hd > (1 << 24) else None
    try:
        base = (2 << 16) + 2 * seq
        k = _draw_matrix(seed, base, L * hkv * n_slots, hd, 1.0, 0.0, dt, pool)
        v = _draw_matrix(seed, base + 1, L * hkv * n_slots, hd, 1.0, 0.0, dt, pool)
    finally:
        if pool is not None:
            pool.shutdown()
    return k.reshape(L, hkv, n_slots, hd), v.reshape(L, hkv, n_slots, hd)


# --------------------------------------------------------------------------------------
# the benchmark configurations (shapes and run parameters only)
# --------------------------------------------------------------------------------------

WORKLOADS = {
    "tiny_fp32": dict(model="tiny", group_policy="packed", group_size=2, gamma=4, context=128, batch=1),
    "llama3_8b_ctx2048": dict(model="llama3_8b", group_policy="aligned", group_size=4, gamma=5,
                              context=2048, batch=1),
    "qwen2_7b_ctx4096": dict(model="qwen2_7b", group_policy="aligned", group_size=4, gamma=5,
                             context=4096, batch=1),
    "llama3_8b_calib_ctx8192": dict(model="llama3_8b", group_policy="aligned", group_size=4, gamma=8,
                                    context=8192, batch=1, calib_tokens="uniform"),
    "llama3_8b_batch4_long": dict(model="llama3_8b", group_policy="aligned", group_size=4, gamma=5,
                                  context=(4096, 8192, 16384, 32768), batch=4),
}
