"""lars_step_ex_static (the LARS step on the library's own fixed scratch array, for callers that cannot allocate)
against lars_step_ex on a caller's workspace: same kernels, so every output must be bit-identical.  Two calls in a
row on the one array, the second with a smaller list, then a third with per-tensor coefficients and a skip list.
The file name sorts last on purpose: the suite is run with -x, and a failure here must not hide other tests."""
import numpy as np
import pytest
import torch

from paper_1709_05011_amd import larsconv as lc
from paper_1709_05011_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
ETA, MOM = 0.001, 0.9


def _device_lists(sizes, seed):
    w = [gu.dev(synth.normal((n,), seed + 3 * i)) for i, n in enumerate(sizes)]
    g = [gu.dev(synth.normal((n,), seed + 3 * i + 1, std=0.01)) for i, n in enumerate(sizes)]
    v = [gu.dev(synth.normal((n,), seed + 3 * i + 2, std=0.001)) for i, n in enumerate(sizes)]
    return w, g, v


def _both_ways(sizes, seed, wd, lr, lowp=False, **per_tensor):
    """One step through each entry point from the same start; returns (reference, static) result tuples."""
    results = []
    for static in (False, True):
        w, g, v = _device_lists(sizes, seed)
        lp = [torch.zeros(n, dtype=torch.int16, device=gu.DEV) for n in sizes] if lowp else None
        args = lc.LarsArgs(w, g, v, list(sizes), lp)
        trust = torch.full((len(sizes),), float("nan"), dtype=torch.float32, device=gu.DEV)
        if static:
            lc.lars_step_ex_static(args, ETA, MOM, wd, lr, trust_out=trust, **per_tensor)
        else:
            ws = gu.workspace(lc.lars_workspace_bytes(args.numel))
            lc.lars_step_ex(args, ETA, MOM, wd, lr, trust_out=trust, workspace=ws, **per_tensor)
        torch.cuda.synchronize()
        results.append((trust.cpu().numpy(), [t.cpu().numpy() for t in w], [t.cpu().numpy() for t in v],
                        [t.cpu().numpy() for t in lp] if lowp else []))
    return results


def _assert_identical(ref, got):
    assert np.array_equal(ref[0].view(np.uint32), got[0].view(np.uint32)), "trust ratios differ"
    assert np.all(np.isfinite(got[0]))
    for a, b in zip(ref[1] + ref[2] + ref[3], got[1] + got[2] + got[3]):
        assert np.array_equal(a, b)


def test_static_scratch_entry_matches_the_workspace_entry_on_two_calls_in_a_row():
    big = synth.resnet50_param_numels()                       # 161 tensors, 25.6 M parameters
    print(f"call 1: {len(big)} tensors, {sum(big)} parameters", flush=True)
    assert lc.lars_workspace_bytes(big) <= lc.LARS_STATIC_SCRATCH_BYTES
    _assert_identical(*_both_ways(big, 900, 5e-5, 0.5))
    small = [1, 63, 4096, 4097, 0, 10000, 3 * 4096 + 5]       # fewer tensors, fewer chunks: the array keeps stale data
    print(f"call 2: {len(small)} tensors, {sum(small)} parameters", flush=True)
    _assert_identical(*_both_ways(small, 901, 5e-4, 1.0, lowp=True))
    n = len(small)
    print("call 3: per-tensor coefficients and a skip list", flush=True)
    _assert_identical(*_both_ways(small, 902, 5e-4, 0.7, eta_per_tensor=[0.001 * (i + 1) for i in range(n)],
                                  weight_decay_per_tensor=[1e-4 * i for i in range(n)], skip=[i % 3 == 1 for i in range(n)]))


def test_static_scratch_entry_refuses_a_list_beyond_its_array():
    # 2 MiB of scratch hold about 420 M parameters; this list asks for more and must be refused before any launch,
    # so the pointers are never used
    numel = [600_000_000]
    assert lc.lars_workspace_bytes(numel) > lc.LARS_STATIC_SCRATCH_BYTES
    fake = [0x10000000]
    args = lc.LarsArgs(fake, fake, fake, numel)
    with pytest.raises(lc.LarsConvError) as e:
        lc.lars_step_ex_static(args, ETA, MOM, 0.0, 1.0, stream=0)
    assert e.value.status == lc.LC_ERR_WORKSPACE
    lc.lars_step_ex_static(lc.LarsArgs([], [], [], []), ETA, MOM, 0.0, 1.0, stream=0)     # empty list: no-op
