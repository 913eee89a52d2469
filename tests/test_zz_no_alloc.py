"""The entry point that allocates nothing (maddness_build_luts_static) against the
entry point it is a variant of (maddness_build_luts), through the C ABI: tables,
scales and offsets bit for bit, on two calls in a row, the second smaller."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mad():
    import torch
    import paper_2106_10860_amd as m
    assert torch.cuda.is_available()
    m.lib()
    return m


def _problem(seed, D, M, C):
    import torch
    rng = np.random.default_rng(seed)
    P = (rng.standard_normal((C, 16, D)) * rng.uniform(0.2, 3.0, size=(C, 1, 1))).astype(np.float32)
    B = (rng.standard_normal((D, M)) / np.sqrt(D)).astype(np.float32)
    params_args = (torch.zeros((C, 4), dtype=torch.int32, device="cuda"),
                   torch.zeros((C, 16), dtype=torch.float32, device="cuda"), torch.from_numpy(P).cuda())
    return params_args, torch.from_numpy(B).cuda()


def test_static_workspace_matches_caller_workspace(mad):
    import torch
    # the second call is smaller than the first: what the first left in the array must not show
    for seed, (D, M, C) in enumerate([(1024, 512, 64), (96, 37, 5), (512, 256, 32)]):
        print("case static workspace", D, M, C, flush=True)
        args, B = _problem(seed, D, M, C)
        params = mad.Params(*args)
        want_luts, want_scale, want_offset = mad.maddness_build_luts(params, B)
        luts = torch.full((C, 16, M), 7, dtype=torch.uint8, device="cuda")
        scale = torch.full((M,), -1.0, device="cuda")
        offset = torch.full((M,), -1.0, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        mad.maddness_build_luts_static(params, B, luts, scale, offset)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(luts, want_luts), "tables differ"
        assert torch.equal(scale.view(torch.int32), want_scale.view(torch.int32)), "scales differ"
        assert torch.equal(offset.view(torch.int32), want_offset.view(torch.int32)), "offsets differ"


def test_static_workspace_rejects_large_tables(mad):
    import torch
    D, M, C = 16, 2048, 64            # 64 * 17 * 2048 doubles: beyond the library's 8 MiB
    args, B = _problem(9, D, M, C)
    params = mad.Params(*args)
    assert mad.lib().maddness_build_luts_workspace(D, C, M) > mad.STATIC_WORKSPACE_BYTES
    luts = torch.zeros((C, 16, M), dtype=torch.uint8, device="cuda")
    scale = torch.zeros(M, device="cuda")
    offset = torch.zeros(M, device="cuda")
    with pytest.raises(mad.MaddnessError) as e:
        mad.maddness_build_luts_static(params, B, luts, scale, offset)
    assert e.value.status == mad.MADDNESS_E_UNSUPPORTED and "workspace" in str(e.value)
