"""bapipe_stage_backward_static (the backward pass on the library's statically allocated workspace,
for callers that cannot allocate device memory) against bapipe_stage_backward, through the C ABI:
same stage, same parameters, same seeded inputs, every output bit for bit - dx of each micro-batch,
losses, and all weight gradients after the mini-batch.  Calls follow one another on the same GPU,
the later ones with smaller inputs, so that whatever a larger stage left in the shared array is there
when the smaller one runs."""
import numpy as np
import pytest

from gpu_harness import GpuStage, gpu_minibatch, stage_io
from paper_2012_12544_amd import binding as B
from stage_inputs import configs as C

pytestmark = pytest.mark.gpu


STAGES = [
    # bottleneck blocks at 24x24: split weight-gradient partials, batch-norm statistics and backward sums handed
    # over through the workspace (above 2048 rows), the dense product of the strided 1x1 input gradient
    ("resnet blocks 24x24", lambda: C.resnet50_stage(cin=64, mid3=32, mid4=64, hw=24, n3=2, n4=2, micro_batch=4, n_micro=3)),
    # the same layers on a quarter of the pixels and fewer samples
    ("resnet blocks 12x12", lambda: C.resnet50_stage(cin=64, mid3=32, mid4=64, hw=12, n3=2, n4=2, micro_batch=3, n_micro=2)),
    ("vgg stage 1, 32x32", lambda: C.vgg16_stage1(c1=64, c2=128, hw=32, micro_batch=2, n_micro=3)),
    ("classifier", lambda: C.vgg16_classifier(c=16, hw=3, hidden=72, classes=13, micro_batch=5, n_micro=3)),
    ("tiny fp32", lambda: C.tiny_stage(c=8, hw=12, micro_batch=2, n_micro=2)),
]


def test_backward_on_the_static_workspace_matches_backward():
    # all static runs first, largest stage first, so that each later call finds the array as the larger one left it
    got = [gpu_minibatch(make(), static=True) for _, make in STAGES]
    for (name, make), a in zip(STAGES, got):
        ref = gpu_minibatch(make(), static=False)
        assert sorted(a) == sorted(ref)
        assert any(k.startswith("dw") for k in ref)
        for k in ref:
            assert np.all(np.isfinite(ref[k])), (name, k)
            assert np.array_equal(a[k], ref[k]), (name, k, float(np.max(np.abs(a[k] - ref[k]))))


def test_static_workspace_rejects_a_stage_that_needs_more():
    """A 1024 -> 1024 3x3 conv splits its weight gradient three ways: 3 x 37.7 MB of partial sums."""
    st = C._stage("wide", [C._layer(C.CONV2D, 1024, 1024, 3, pad=1, has_bias=1, src0=-1)], C.BF16, (1024, 28, 28),
                  4, 1, 1, 1, 1, C.BASE_SEED + 5, "kaiming")
    g = GpuStage(st, [(None, None)])
    xs, gs = stage_io(st)
    g.forward(0, xs[0])
    with pytest.raises(B.BapipeError) as e:
        g.backward(0, gs[0], static=True)
    assert e.value.status == B.E_UNSUPPORTED and "workspace" in str(e.value)
    dx = g.backward(0, gs[0])                   # nothing was enqueued or changed: the ordinary call still runs
    assert dx.shape == xs[0].shape and not dx.any()      # weights are still zero
    g.close()
