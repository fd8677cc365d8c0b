"""The entry point that allocates nothing (dhq_forward_noalloc) against dhq_forward with
DHQ_DYNAMIC, which runs the same kernels on buffers the model allocates: same bits, on two calls
in a row of which the second brings fewer rows (the fixed scratch buffer then still holds the
first call's data).  Every call goes through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2508_13478_amd as dhq
from paper_2508_13478_amd import synth

pytestmark = pytest.mark.gpu


def _coords(n, k, seed):
    return synth.uniform(seed, 0, n * k, -1.0, 1.0).reshape(n, k)


CASES = [
    # dims, mode, flags, rows of the two calls
    ((2, 64, 64, 64, 3), dhq.DHQ_ROTATE_IN, dhq.DHQ_FUSED, (4096, 1000)),
    ((2, 256, 256, 256, 256, 3), dhq.DHQ_ROTATE_IN, dhq.DHQ_AUTO, (14336, 777)),
    ((2, 256, 256, 256, 256, 3), dhq.DHQ_ROTATE_IN, dhq.DHQ_LAYERWISE, (9000, 8999)),
    ((2, 128, 128, 3), dhq.DHQ_ROTATE_BOTH, dhq.DHQ_FUSED, (5001, 33)),
    ((3, 100, 48, 5), dhq.DHQ_ROTATE_BOTH, dhq.DHQ_LAYERWISE, (3001, 1)),
    ((2, 512, 512, 3), dhq.DHQ_ROTATE_IN, dhq.DHQ_AUTO, (7000, 6000)),
]


@pytest.mark.parametrize("dims,mode,flags,rows", CASES)
def test_noalloc_matches_dynamic_forward(dims, mode, flags, rows):
    W, b = synth.siren_init(list(dims), 30.0, 0xA110C + len(dims) + dims[1])
    model = dhq.Model(dims, 30.0, W, b, 8, 8, mode=mode)
    assert dhq.dhq_noalloc_max_rows(model.handle) >= max(rows)
    for i, n in enumerate(rows):
        x = torch.from_numpy(_coords(n, dims[0], 0xC0 + i)).to("cuda")
        ref = torch.empty((n, dims[-1]), dtype=torch.float32, device="cuda")
        got = torch.full((n, dims[-1]), float("nan"), dtype=torch.float32, device="cuda")
        dhq.dhq_forward(model.handle, x, ref, None, flags | dhq.DHQ_DYNAMIC)
        s_ref = model.dynamic_scales()
        dhq.dhq_forward_noalloc(model.handle, x, got, None, flags)
        s_got = model.dynamic_scales()
        torch.cuda.synchronize()
        assert torch.equal(got, ref), (dims, n, float((got - ref).abs().max()))
        assert np.array_equal(s_ref, s_got)
    model.close()


def test_noalloc_rejects_what_does_not_fit():
    dims = (2, 256, 256, 3)
    W, b = synth.siren_init(list(dims), 30.0, 7)
    model = dhq.Model(dims, 30.0, W, b, 8, 8)
    cap = dhq.dhq_noalloc_max_rows(model.handle)
    assert 14336 <= cap < (1 << 22)
    n = cap + 1
    x = torch.zeros((n, 2), dtype=torch.float32, device="cuda")
    out = torch.zeros((n, 3), dtype=torch.float32, device="cuda")
    with pytest.raises(dhq.DhqError) as e:
        dhq.dhq_forward_noalloc(model.handle, x, out, None, dhq.DHQ_AUTO)
    assert e.value.status == dhq.DHQ_ETOOBIG
    with pytest.raises(dhq.DhqError) as e:
        dhq.dhq_forward_noalloc(model.handle, x[:8], out[:8], None, dhq.DHQ_DYNAMIC)   # not a path flag
    assert e.value.status == dhq.DHQ_EINVAL
    dhq.dhq_forward_noalloc(model.handle, x[:0], out[:0], None, dhq.DHQ_AUTO)         # nothing to do
    # the largest size it takes still runs
    dhq.dhq_forward_noalloc(model.handle, x[:cap], out[:cap], None, dhq.DHQ_AUTO)
    torch.cuda.synchronize()
    ref = torch.empty_like(out[:cap])
    dhq.dhq_forward(model.handle, x[:cap], ref, None, dhq.DHQ_AUTO | dhq.DHQ_DYNAMIC)
    torch.cuda.synchronize()
    assert torch.equal(out[:cap], ref)
    model.close()
    fl = dhq.Model(dims, 30.0, W, b, 8, 8, mode=dhq.DHQ_W32A32)
    assert dhq.dhq_noalloc_max_rows(fl.handle) == 0
    fl.close()
