"""The allocation-free acceptance entry point (easyspec_accept_static: the library's own fixed device
array as workspace) against easyspec_accept with a caller's workspace, through the C ABI: accept
lengths and bonus tokens are integers and must be equal, on two calls in a row of which the second
is smaller (it finds the first call's contents in the shared array).  Collected last on purpose."""
import numpy as np
import pytest

from test_gpu_accept import make_case

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def es():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device; none is visible")
    import paper_2502_02493_amd as es
    return es


def both(es, case, T, stream=None, first_call=False):
    """first_call: the very first launch of a process may load the library's code object (and with it
    the fixed array), which is not an allocation of the call."""
    import torch
    draft, dl, tl, r, u = case
    batch, gamma = draft.shape
    V = tl.shape[-1]
    dev = torch.device("cuda:0")
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    d_draft, d_dl, d_tl, d_r, d_u = t(draft), t(dl), t(tl), t(r), t(u)
    out = []
    ws = torch.empty(es.easyspec_accept_workspace_bytes(batch, gamma, V) // 8, dtype=torch.float64, device=dev)
    handle = torch.cuda.current_stream().cuda_stream if stream is None else stream.cuda_stream
    for static in (False, True):
        acc = torch.full((batch,), -7, dtype=torch.int32, device=dev)
        bon = torch.full((batch,), -7, dtype=torch.int32, device=dev)
        torch.cuda.synchronize()
        before = torch.cuda.mem_get_info()[0]                 # free device memory as the driver sees it
        if static:
            es.easyspec_accept_static(d_draft, d_dl, d_tl, d_r, d_u, batch, gamma, V, T, acc, bon, handle)
        else:
            es.easyspec_accept(d_draft, d_dl, d_tl, d_r, d_u, batch, gamma, V, T, acc, bon, ws, handle)
        torch.cuda.synchronize()
        if static and not first_call:
            assert torch.cuda.mem_get_info()[0] == before, "the call changed the device's free memory"
        out.append((acc.cpu().numpy(), bon.cpu().numpy()))
    return out


def test_static_workspace_equals_caller_workspace_twice_in_a_row(oracle, es):
    assert es.easyspec_accept_static_max_bytes() == 8 << 20
    first = make_case(4001, 4, 5, 128256, 0.8, 0.7)          # 4 sequences at the 8B shape's vocabulary: 4.1 MB of workspace
    second = make_case(4002, 2, 3, 1031, 0.8, 1.0)           # smaller: the array still holds the first call's numbers
    third = make_case(4003, 6, 5, 152064, 0.8, 0.5)          # the largest that fits (Qwen2-7B's vocabulary): 7.3 MB
    for i, case in enumerate((first, second, third, second)):
        (a0, b0), (a1, b1) = both(es, case, 0.8, first_call=i == 0)
        assert np.array_equal(a0, a1) and np.array_equal(b0, b1)
        assert np.all(a0 >= 0) and np.all(b0 >= 0)
        draft, dl, tl, r, u = case
        for b in range(draft.shape[0]):                      # and both equal the oracle
            m, bonus, margin = oracle.accept(draft[b], dl[b], tl[b], r[b], u[b], 0.8, with_margin=True)
            if margin > 1e-9:
                assert (int(a1[b]), int(b1[b])) == (m, bonus)


def test_static_workspace_on_a_second_stream_and_bad_token(es):
    import torch
    case = make_case(4004, 3, 4, 4099, 0.8, 0.7)
    case[0][1, 0] = 4099                                      # not a token: that sequence reports -1, -1
    (a0, b0), (a1, b1) = both(es, case, 0.8, stream=torch.cuda.Stream())
    assert np.array_equal(a0, a1) and np.array_equal(b0, b1)
    assert a1[1] == -1 and b1[1] == -1 and a1[0] >= 0


def test_static_workspace_refuses_what_does_not_fit(es):
    import torch
    dev = torch.device("cuda:0")
    batch, gamma, V = 7, 5, 152064
    assert es.easyspec_accept_workspace_bytes(batch, gamma, V) > es.easyspec_accept_static_max_bytes()
    z = torch.zeros(8, dtype=torch.int32, device=dev)        # never dereferenced: the size check comes first
    with pytest.raises(es.EasySpecError) as e:
        es.easyspec_accept_static(z, z, z, z, z, batch, gamma, V, 0.8, z, z, None)
    assert e.value.code == es.EASYSPEC_ECAPACITY and "workspace" in str(e.value)
    with pytest.raises(es.EasySpecError) as e:
        es.easyspec_accept_static(z, z, z, z, z, 1, 5, 1000, 0.0, z, z, None)
    assert e.value.code == es.EASYSPEC_EINVAL
