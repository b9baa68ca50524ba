"""Test-side convenience around the C-ABI binding: owns torch device buffers for token ids and
logits and converts results to numpy.  Every computation goes through libeasyspec.so."""
from __future__ import annotations

import os

import numpy as np
import torch

import easyspec_synth as synth
import paper_2502_02493_amd as es


from tolerances import FULL_SIZE_TOL, MARGIN, PEAK_PER_TOL, PLAIN_TOL, TOL  # noqa: F401

_LOG = os.environ.get("EASYSPEC_PARITY_LOG")


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def peak_dev(a, b):
    """Largest |a - b| in units of rms(b)."""
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    rms = max(float(np.linalg.norm(b)) / np.sqrt(b.size), 1e-300)
    return float(np.max(np.abs(a - b))) / rms


def assert_close(got, want, tol, what=""):
    """rel-L2 below tol and no single element further than PEAK_PER_TOL * tol * rms(want) from the oracle."""
    err, peak = rel_l2(got, want), peak_dev(got, want)
    if _LOG:
        with open(_LOG, "a") as f:
            f.write(f"{err:.3e} {peak:.3e} {tol:.1e} {np.asarray(want).size} {os.environ.get('PYTEST_CURRENT_TEST', '?')} | {what}\n")
    assert err < tol, f"{what}: rel-L2 {err:.3e} >= {tol:.1e}"
    assert peak < PEAK_PER_TOL * tol, f"{what}: largest deviation {peak:.3e} rms >= {PEAK_PER_TOL * tol:.1e}"
    return err


class GpuDrafter:
    def __init__(self, cfg: dict, weights: dict, max_batch=1, max_ctx=256, max_calib=16, stream=None):
        assert torch.cuda.is_available()
        self.cfg, self.B, self.max_ctx, self.mc = cfg, max_batch, max_ctx, max_calib
        self.dev = torch.device("cuda:0")
        self.ctx = es.easyspec_create(es.make_config(cfg, max_batch, max_ctx, max_calib), stream)
        es.easyspec_load_weights(self.ctx, weights)
        V = cfg["vocab"]
        self.tok_in = torch.zeros(max_batch, dtype=torch.int32, device=self.dev)
        self.tok_out = torch.full((max_batch,), -1, dtype=torch.int32, device=self.dev)
        self.logits = torch.zeros(max_batch, V, dtype=torch.float32, device=self.dev)
        self.calib_tok = torch.zeros(max_batch, max_calib, dtype=torch.int32, device=self.dev)
        self.calib_logits = torch.zeros(max_batch, max_calib, V, dtype=torch.float32, device=self.dev)

    def close(self):
        if self.ctx is not None:
            es.easyspec_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_groups(self, bounds):
        es.easyspec_set_groups(self.ctx, bounds)

    def set_full_layer(self, on: bool):
        es.easyspec_set_parallel_mode(self.ctx, es.EASYSPEC_PARALLEL_FULL_LAYER if on else es.EASYSPEC_PARALLEL_ATTENTION)

    def lens(self):
        return es.easyspec_get_lens(self.ctx, self.B)

    def calibrate(self, tokens_by_seq: dict, all_rows=True):
        """tokens_by_seq: {b: [ids]} with 1..max_calib ids each.  Returns ({b: next id}, {b: logits})
        where logits is [n, V] (all_rows) or [V]."""
        n = np.zeros(self.B, np.int32)
        host = np.zeros((self.B, self.mc), np.int32)
        for b, t in tokens_by_seq.items():
            n[b] = len(t)
            host[b, : len(t)] = t
        self.calib_tok.copy_(torch.from_numpy(host))
        self.tok_out.fill_(-1)
        if all_rows:
            es.easyspec_calibrate(self.ctx, self.calib_tok, n, self.tok_out, self.calib_logits, 1)
        else:
            es.easyspec_calibrate(self.ctx, self.calib_tok, n, self.tok_out, self.logits, 0)
        torch.cuda.synchronize()
        toks = self.tok_out.cpu().numpy()
        if all_rows:
            lg = self.calib_logits.cpu().numpy()
            return {b: int(toks[b]) for b in tokens_by_seq}, {b: lg[b, : n[b]].copy() for b in tokens_by_seq}
        lg = self.logits.cpu().numpy()
        return {b: int(toks[b]) for b in tokens_by_seq}, {b: lg[b].copy() for b in tokens_by_seq}

    def prefill(self, b: int, prompt):
        """Chunked calibration of a prompt; returns (next id, logits [len, V])."""
        rows, nxt = [], None
        for i in range(0, len(prompt), self.mc):
            t, lg = self.calibrate({b: list(prompt[i: i + self.mc])})
            rows.append(lg[b])
            nxt = t[b]
        return nxt, np.concatenate(rows)

    def draft_step(self, tokens_by_seq: dict):
        host = np.zeros(self.B, np.int32)
        for b, t in tokens_by_seq.items():
            host[b] = t
        self.tok_in.copy_(torch.from_numpy(host))
        self.tok_out.fill_(-1)
        es.easyspec_draft_step(self.ctx, self.tok_in, self.tok_out, self.logits)
        torch.cuda.synchronize()
        return self.tok_out.cpu().numpy().copy(), self.logits.cpu().numpy().copy()

    def draft_tree_step(self, nodes_by_seq: dict):
        """nodes_by_seq: {b: ([token ids], [parents])}.  Returns ({b: argmax ids [n]}, {b: logits [n, V]})."""
        W, V = es.EASYSPEC_MAX_TREE_WIDTH, self.cfg["vocab"]
        if not hasattr(self, "tree_in"):
            self.tree_in = torch.zeros(self.B, W, dtype=torch.int32, device=self.dev)
            self.tree_out = torch.zeros(self.B, W, dtype=torch.int32, device=self.dev)
            self.tree_logits = torch.zeros(self.B, W, V, dtype=torch.float32, device=self.dev)
        n = np.zeros(self.B, np.int32)
        host = np.zeros((self.B, W), np.int32)
        par = np.full((self.B, W), -1, np.int32)
        for b, (t, p) in nodes_by_seq.items():
            n[b] = len(t)
            host[b, : len(t)] = t
            par[b, : len(p)] = p
        self.tree_in.copy_(torch.from_numpy(host))
        self.tree_out.fill_(-1)
        es.easyspec_draft_tree_step(self.ctx, self.tree_in, n, par, self.tree_out, self.tree_logits)
        torch.cuda.synchronize()
        toks, lg = self.tree_out.cpu().numpy(), self.tree_logits.cpu().numpy()
        return ({b: toks[b, : n[b]].copy() for b in nodes_by_seq}, {b: lg[b, : n[b]].copy() for b in nodes_by_seq})

    def hidden(self):
        out = torch.zeros(16, self.cfg["d_model"], dtype=torch.float32, device=self.dev)
        n = es.easyspec_get_hidden(self.ctx, out, 16)
        torch.cuda.synchronize()
        return out[:n].cpu().numpy()

    def export_kv(self, b: int, n: int):
        """float32 arrays [L, Hkv, n, hd]."""
        c = self.cfg
        shape = (c["n_layers"], c["n_kv_heads"], n, c["head_dim"])
        dt = np.uint16 if c["dtype"] == "bf16" else np.float32
        k, v = np.zeros(shape, dt), np.zeros(shape, dt)
        es.easyspec_kv_export(self.ctx, b, k, v, n)
        if dt == np.uint16:
            k, v = synth.bf16_bits_to_f32(k).reshape(shape), synth.bf16_bits_to_f32(v).reshape(shape)
        return k, v

    def import_kv(self, b: int, k, v):
        es.easyspec_kv_import(self.ctx, b, np.ascontiguousarray(k), np.ascontiguousarray(v), k.shape[2])
