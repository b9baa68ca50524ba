"""GPU tests of the state machine around the kernels: the lossless greedy loop, error
handling (host-forced, no kernel misbehaves), dropped fuzzy slots, determinism, device-side
greedy acceptance."""
import itertools

import numpy as np
import pytest

import easyspec_synth as synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device; none is visible")
    import gpu_harness
    return gpu_harness


@pytest.mark.parametrize("bounds", [[0, 1, 3, 4], [0, 4], [0, 1, 2, 3, 4]])
def test_lossless_greedy_loop_on_gpu(oracle, gpu, bounds):
    """Three-stage loop with the drafter AND a tiny base model both on the GPU (the base model is
    a second context run in sequential order through easyspec_calibrate with all-row logits):
    the output equals the oracle's vanilla greedy decoding of the base model token for token."""
    import paper_2502_02493_amd as es
    cfg = synth.model_shape("tiny")
    wd, wb = synth.make_weights(cfg, 600), synth.make_weights(cfg, 601)
    prompt = [int(t) for t in synth.make_tokens(602, 24, cfg["vocab"])]
    gamma, n_new = 4, 40
    base_o = oracle.Sequence(oracle.Model(cfg, wb, 128))
    want = oracle.vanilla_greedy(base_o, prompt, n_new)

    d = gpu.GpuDrafter(cfg, wd, 1, 128, 16)
    b = gpu.GpuDrafter(cfg, wb, 1, 128, 16)
    try:
        d.set_groups(bounds)
        out, accepts = [], []
        b.prefill(0, prompt[:-1])
        last, calib = prompt[-1], list(prompt)
        while len(out) < n_new:
            nxt = None
            for i in range(0, len(calib), 16):                       # first round: the prompt, in chunks
                t, _ = d.calibrate({0: calib[i:i + 16]}, all_rows=False)
                nxt = t[0]
            drafted = [nxt]
            for _ in range(gamma - 1):
                t, _ = d.draft_step({0: drafted[-1]})
                drafted.append(int(t[0]))
            p0 = int(b.lens()[0][0])
            _, vl = b.calibrate({0: [last] + drafted}, all_rows=True)
            target = np.argmax(vl[0], axis=1).astype(np.int32)       # the verifier's greedy choices
            acc, bonus = np.zeros(1, np.int32), np.zeros(1, np.int32)
            es.easyspec_greedy_accept_host(np.array(drafted, np.int32), target, 1, gamma, acc, bonus)
            m = int(acc[0])
            es.easyspec_truncate(b.ctx, 0, p0 + 1 + m)
            accepts.append(m)
            out.extend(drafted[:m] + [int(bonus[0])])
            calib, last = drafted[:m] + [int(bonus[0])], int(bonus[0])
        assert out[:n_new] == want
        p, f = d.lens()
        assert int(f[0]) == 0 or int(f[0]) == gamma - 1
    finally:
        d.close(); b.close()


def test_self_draft_accepts_everything_on_gpu(oracle, gpu):
    """Draft weights = base weights and all sets of size one: the fuzzy step is the sequential
    step, so every drafted token is accepted."""
    import paper_2502_02493_amd as es
    cfg = synth.model_shape("tiny")
    w = synth.make_weights(cfg, 610)
    prompt = [int(t) for t in synth.make_tokens(611, 16, cfg["vocab"])]
    d, b = gpu.GpuDrafter(cfg, w, 1, 96, 16), gpu.GpuDrafter(cfg, w, 1, 96, 16)
    try:
        b.prefill(0, prompt[:-1])
        last, calib, gamma = prompt[-1], list(prompt), 4
        for _ in range(6):
            t, _ = d.calibrate({0: calib}, all_rows=False)
            drafted = [t[0]]
            for _ in range(gamma - 1):
                tt, _ = d.draft_step({0: drafted[-1]})
                drafted.append(int(tt[0]))
            p0 = int(b.lens()[0][0])
            _, vl = b.calibrate({0: [last] + drafted}, all_rows=True)
            target = np.argmax(vl[0], axis=1).astype(np.int32)
            acc, bonus = np.zeros(1, np.int32), np.zeros(1, np.int32)
            es.easyspec_greedy_accept_host(np.array(drafted, np.int32), target, 1, gamma, acc, bonus)
            assert int(acc[0]) == gamma
            es.easyspec_truncate(b.ctx, 0, p0 + 1 + gamma)
            calib, last = drafted + [int(bonus[0])], int(bonus[0])
    finally:
        d.close(); b.close()


def test_error_paths_leave_state_unchanged(gpu):
    import torch
    import paper_2502_02493_amd as es
    cfg = synth.model_shape("tiny")
    w = synth.make_weights(cfg, 620)
    dev = torch.device("cuda:0")
    ctx = es.easyspec_create(es.make_config(cfg, 2, 12, 4), None)
    try:
        tok = torch.zeros(2, 4, dtype=torch.int32, device=dev)
        one = torch.zeros(2, dtype=torch.int32, device=dev)

        def code(fn, *a):
            with pytest.raises(es.EasySpecError) as e:
                fn(*a)
            return e.value.code

        assert code(es.easyspec_draft_step, ctx, one, one, None) == es.EASYSPEC_ESTATE            # no weights yet
        assert code(es.easyspec_calibrate, ctx, tok, [1, 0], one, None, 0) == es.EASYSPEC_ESTATE
        es.easyspec_load_weights(ctx, w)
        assert code(es.easyspec_draft_step, ctx, one, one, None) == es.EASYSPEC_ESTATE            # nothing live yet
        assert "no live sequence" in es.easyspec_last_error(ctx)
        assert code(es.easyspec_calibrate, ctx, tok, [5, 0], one, None, 0) == es.EASYSPEC_ECAPACITY  # > max_calib_tokens
        assert code(es.easyspec_calibrate, ctx, tok, [0, 0], one, None, 0) == es.EASYSPEC_EINVAL
        assert code(es.easyspec_calibrate, ctx, tok, [1, 0], one, None, 2) == es.EASYSPEC_EINVAL
        assert code(es.easyspec_calibrate, ctx, None, [1, 0], one, None, 0) == es.EASYSPEC_EINVAL
        assert code(es.easyspec_set_groups, ctx, [0, 2, 2, 4]) == es.EASYSPEC_EINVAL
        assert code(es.easyspec_set_groups, ctx, [0, 2, 3]) == es.EASYSPEC_EINVAL
        assert code(es.easyspec_set_groups, ctx, [1, 2, 4]) == es.EASYSPEC_EINVAL
        es.easyspec_set_groups(ctx, [0, 1, 3, 4])
        for _ in range(3):
            es.easyspec_calibrate(ctx, tok, [4, 0], one, None, 0)                                   # 12 of 12 slots
        p, f = es.easyspec_get_lens(ctx, 2)
        assert list(p) == [12, 0] and list(f) == [0, 0]
        assert code(es.easyspec_draft_step, ctx, one, one, None) == es.EASYSPEC_ECAPACITY         # sequence 0 is full
        assert code(es.easyspec_calibrate, ctx, tok, [1, 0], one, None, 0) == es.EASYSPEC_ECAPACITY
        p2, f2 = es.easyspec_get_lens(ctx, 2)
        assert list(p2) == [12, 0] and list(f2) == [0, 0]                                           # nothing moved
        assert code(es.easyspec_truncate, ctx, 0, 13) == es.EASYSPEC_EINVAL
        assert code(es.easyspec_truncate, ctx, 2, 1) == es.EASYSPEC_EINVAL
        es.easyspec_truncate(ctx, 0, 10)
        es.easyspec_draft_step(ctx, one, one, None)
        es.easyspec_draft_step(ctx, one, one, None)
        assert code(es.easyspec_draft_step, ctx, one, one, None) == es.EASYSPEC_ECAPACITY
        p, f = es.easyspec_get_lens(ctx, 2)
        assert list(p) == [10, 0] and list(f) == [2, 0]
        k = np.zeros((4, 2, 13, 64), np.float32)
        assert code(es.easyspec_kv_import, ctx, 0, k, k, 13) == es.EASYSPEC_ECAPACITY
        assert code(es.easyspec_kv_import, ctx, 5, k, k, 3) == es.EASYSPEC_EINVAL
        assert code(es.easyspec_profile_end, ctx) == es.EASYSPEC_ESTATE
        torch.cuda.synchronize()
    finally:
        es.easyspec_destroy(ctx)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_dropped_fuzzy_slots_are_never_read(gpu, dtype):
    """After calibration the slots beyond the precise length are dead: filling them with NaN
    changes no later result bit."""
    cfg = synth.model_shape("tiny", dtype=dtype)
    w = synth.make_weights(cfg, 630)
    toks = [int(t) for t in synth.make_tokens(631, 32, cfg["vocab"])]
    bounds = [0, 1, 3, 4]

    def run(poison):
        g = gpu.GpuDrafter(cfg, w, 1, 64, 16)
        try:
            g.set_groups(bounds)
            g.calibrate({0: toks[:9]})
            for t in toks[9:13]:
                g.draft_step({0: t})                                   # 4 fuzzy slots
            if poison:
                k, v = g.export_kv(0, 13)
                k[:, :, 9:] = np.nan; v[:, :, 9:] = np.nan
                if dtype == "bf16":
                    k, v = synth.f32_to_bf16_bits(np.nan_to_num(k, nan=0.0)).reshape(k.shape), \
                        synth.f32_to_bf16_bits(np.nan_to_num(v, nan=0.0)).reshape(v.shape)
                    k[:, :, 9:] = 0x7FC0; v[:, :, 9:] = 0x7FC0       # bf16 quiet NaN
                import paper_2502_02493_amd as es
                g.import_kv(0, k, v)
                es.easyspec_truncate(g.ctx, 0, 9)
            _, l1 = g.calibrate({0: toks[13:15]})                      # accepts 1 token + bonus
            _, l2 = g.draft_step({0: toks[15]})
            return l1[0], l2[0]
        finally:
            g.close()

    a1, a2 = run(False)
    b1, b2 = run(True)
    assert np.all(np.isfinite(b1)) and np.all(np.isfinite(b2))
    assert np.array_equal(a1, b1) and np.array_equal(a2, b2)


@pytest.mark.parametrize("shape,dtype,bounds", [("tiny", "fp32", [0, 1, 3, 4]), ("tiny", "bf16", [0, 4]),
                                                ("tiny_qwen", "bf16", [0, 1, 4, 5])])
def test_workspaces_hold_nothing_between_calls(gpu, monkeypatch, shape, dtype, bounds):
    """Every workspace between the kernels of a pass (residual stream, norm operands and partial sums,
    queries, attention outputs, split-KV partials, parked Attnoutputs, MLP activations, argmax candidates)
    is filled with NaN before every call: logits, drafted ids and the cache keep every bit.  Covers
    prefill in chunks, split-KV attention with a merge (context beyond one chunk), chain steps, a tree
    level on the vector kernel and on the matrix cores, a two-fragment calibration, and the full-layer mode."""
    import paper_2502_02493_amd as es
    cfg = synth.model_shape(shape, dtype=dtype)
    w = synth.make_weights(cfg, 650)
    toks = [int(t) for t in synth.make_tokens(651, 400, cfg["vocab"])]

    def run(poison):
        g = gpu.GpuDrafter(cfg, w, 2, 512, 16)
        outs = []

        def p():
            if poison:
                es.easyspec_poison_workspaces(g.ctx)

        try:
            g.set_groups(bounds)
            for i in range(0, 320, 16):                                   # 320 slots: past the single-chunk limit
                p(); _, l = g.calibrate({0: toks[i:i + 16]})
            outs.append(l[0])
            p(); _, l = g.calibrate({1: toks[320:331]}); outs.append(l[1])   # 11 columns: two activation fragments (bf16)
            for t in toks[331:334]:
                p(); tk, l = g.draft_step({0: t, 1: t + 1 if t + 1 < cfg["vocab"] else 0}); outs += [tk.copy(), l]
            p(); _, l = g.calibrate({0: toks[334:337]}); outs.append(l[0])
            p(); tk, l = g.draft_tree_step({0: (toks[337:341], [-1, -1, -1, -1])}); outs += [tk[0], l[0]]
            p(); tk, l = g.draft_tree_step({0: (toks[341:347], [0, 0, 1, 2, 3, 3])}); outs += [tk[0], l[0]]
            g.set_full_layer(True)
            p(); _, l = g.calibrate({0: toks[347:349], 1: toks[349:350]}); outs += [l[0], l[1]]
            p(); tk, l = g.draft_step({0: toks[350], 1: toks[351]}); outs += [tk.copy(), l]
            k, v = g.export_kv(0, int(g.lens()[0][0]) + int(g.lens()[1][0]))
            outs += [k, v]
            return outs
        finally:
            g.close()

    a = run(False)
    for mfma in ("1", "2"):                                               # 2: every multi-column launch on the matrix cores (bf16)
        monkeypatch.setenv("EASYSPEC_ATTN_MFMA", mfma)
        ref = a if mfma == "1" else run(False)
        b = run(True)
        assert len(ref) == len(b)
        for x, y in zip(ref, b):
            assert np.all(np.isfinite(np.asarray(y, dtype=np.float64)))
            assert np.array_equal(x, y)


def test_per_launch_timing_counts_every_launch(gpu):
    """easyspec_profile_*: every launch of the profiled kernel class carries its own event pair; the count is
    the launch count the set table implies and every duration is a plausible kernel time."""
    import paper_2502_02493_amd as es
    cfg = synth.model_shape("tiny")
    w = synth.make_weights(cfg, 660)
    g = gpu.GpuDrafter(cfg, w, 1, 600, 16)
    try:
        g.set_groups([0, 1, 3, 4])
        toks = [int(t) for t in synth.make_tokens(661, 330, cfg["vocab"])]
        for i in range(0, 320, 16):
            g.calibrate({0: toks[i:i + 16]})
        _, ref = g.draft_step({0: toks[320]})
        es.easyspec_truncate(g.ctx, 0, 320)
        want = {es.EASYSPEC_OP_QKV: 3, es.EASYSPEC_OP_ATTN: 6, es.EASYSPEC_OP_OPROJ: 3, es.EASYSPEC_OP_GATEUP: 4,
                es.EASYSPEC_OP_DOWN: 4, es.EASYSPEC_OP_HEAD: 2}             # 3 sets, 4 layers; attention = partial + merge
        for op, n_want in want.items():
            per = np.full(16, -1.0, np.float32)
            es.easyspec_profile_begin(g.ctx, op, 16)
            _, got = g.draft_step({0: toks[320]})
            n, total = es.easyspec_profile_end(g.ctx, per)
            es.easyspec_truncate(g.ctx, 0, 320)
            assert n == n_want, (op, n)
            assert np.all(per[:n] > 0.0005) and np.all(per[:n] < 1.0) and np.all(per[n:] == -1.0), per    # 0.5 us ... 1 ms
            assert abs(float(per[:n].sum()) - total) < 1e-3 * total + 1e-6
            assert np.array_equal(got, ref)                                 # timing changes no result
        # every kernel of the pass, with its class, in launch order: embed; per set QKV, attention, merge, O, then
        # gate/up and down per layer; head and argmax
        per, ops = np.zeros(64, np.float32), np.full(64, -1, np.int32)
        es.easyspec_profile_begin(g.ctx, es.EASYSPEC_OP_ALL, 64)
        _, got = g.draft_step({0: toks[320]})
        n, total = es.easyspec_profile_end(g.ctx, per, ops)
        es.easyspec_truncate(g.ctx, 0, 320)
        Q, A, O, G, D, H, E = (es.EASYSPEC_OP_QKV, es.EASYSPEC_OP_ATTN, es.EASYSPEC_OP_OPROJ, es.EASYSPEC_OP_GATEUP,
                               es.EASYSPEC_OP_DOWN, es.EASYSPEC_OP_HEAD, es.EASYSPEC_OP_ALL)
        assert list(ops[:n]) == [E, Q, A, A, O, G, D, Q, A, A, O, G, D, G, D, Q, A, A, O, G, D, H, H]
        assert np.all(per[:n] > 0.0005) and np.array_equal(got, ref)
        es.easyspec_profile_begin(g.ctx, es.EASYSPEC_OP_GATEUP, 2)          # fewer pairs than launches: the rest runs untimed
        g.draft_step({0: toks[320]})
        n, _ = es.easyspec_profile_end(g.ctx)
        assert n == 2
    finally:
        g.close()


def test_repeated_runs_are_bit_identical(gpu):
    """Fixed summation orders everywhere: the same calls give the same bits."""
    cfg = synth.model_shape("tiny_qwen", dtype="bf16")
    w = synth.make_weights(cfg, 640)
    toks = [int(t) for t in synth.make_tokens(641, 40, cfg["vocab"])]
    outs = []
    for _ in range(2):
        g = gpu.GpuDrafter(cfg, w, 2, 96, 16)
        try:
            g.set_groups([0, 1, 4, 5])
            _, l0 = g.calibrate({0: toks[:16], 1: toks[16:21]})
            _, l1 = g.draft_step({0: toks[21], 1: toks[22]})
            outs.append((l0[0], l0[1], l1))
        finally:
            g.close()
    for a, b in zip(outs[0], outs[1]):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("which_stream", ["default", "side"])
def test_greedy_accept_device_path(oracle, gpu, which_stream):
    """The acceptance kernel on the default stream (handle 0) and on a second stream.  The outputs are
    poisoned on the device beforehand and the inputs are produced by device work queued on the same
    stream right before the call, so only a kernel ordered on that stream can give the right answer."""
    import torch
    import paper_2502_02493_amd as es
    dev = torch.device("cuda:0")
    gamma = 3
    pairs = list(itertools.product(itertools.product(range(3), repeat=gamma), itertools.product(range(3), repeat=gamma + 1)))
    d_host = torch.tensor([p[0] for p in pairs], dtype=torch.int32)
    t_host = torch.tensor([p[1] for p in pairs], dtype=torch.int32)
    stream = torch.cuda.current_stream() if which_stream == "default" else torch.cuda.Stream()
    if which_stream == "default":
        assert stream.cuda_stream == 0
    with torch.cuda.stream(stream):
        acc = torch.full((len(pairs),), -77, dtype=torch.int32, device=dev)
        bonus = torch.full((len(pairs),), -77, dtype=torch.int32, device=dev)
        # the inputs reach their final values through a chain of device work on this stream
        big = torch.zeros(1 << 24, dtype=torch.int32, device=dev)
        for _ in range(4):
            big += 1
        d = d_host.to(dev) + big[: d_host.numel()].view_as(d_host) - 4
        t = t_host.to(dev) + big[: t_host.numel()].view_as(t_host) - 4
        es.easyspec_greedy_accept(d, t, len(pairs), gamma, acc, bonus, stream.cuda_stream)
        stream.synchronize()
    acc, bonus = acc.cpu().numpy(), bonus.cpu().numpy()
    assert not np.any(acc == -77) and not np.any(bonus == -77)
    for i, (dd, tt) in enumerate(pairs):
        assert (int(acc[i]), int(bonus[i])) == oracle.greedy_accept(dd, tt)
    # host arrays are refused, not looped over on the host
    with pytest.raises(es.EasySpecError):
        es.easyspec_greedy_accept(d_host.numpy(), t_host.numpy(), len(pairs), gamma, np.zeros(len(pairs), np.int32),
                                  np.zeros(len(pairs), np.int32), stream.cuda_stream)
