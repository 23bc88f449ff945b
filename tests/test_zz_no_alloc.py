"""xenos_run_static: the entry point that allocates nothing (the intermediate tensors live in a device array that is
part of the library's image) against xenos_run with a caller-provided workspace, through the C ABI."""
import numpy as np
import pytest

from workloads import cnn_graphs as wg

pytestmark = pytest.mark.gpu


def _xenos():
    from paper_2302_00282_amd import xenos as X
    X.lib()
    return X


def _both(X, g, compute, link):
    """(output of xenos_run with a bound workspace, output of xenos_run_static with none bound)"""
    s = X.Session(g, link=link, compute=compute)
    try:
        want = s.forward(g.x).copy()
        need = s.info["workspace_bytes"]
    finally:
        s.close()
    t = X.Session(g, link=link, compute=compute, workspace=False)
    try:
        t.set_input(g.x)
        t.y.fill_(float("nan"))
        t.run_static()
        got = t.output().copy()
        with pytest.raises(X.XenosError):                     # no workspace bound: the other run calls refuse
            t.run()
    finally:
        t.close()
    return want, got, need


@pytest.mark.parametrize("compute", [1, 0])
def test_static_workspace_run_equals_run_twice_in_a_row(compute):
    X = _xenos()
    big = wg.resnet18(batch=3, hw=96, width=0.5, classes=24, seed=71, nonzero_bias=True)
    small = wg.mobilenet_v1(batch=1, hw=64, width=0.25, classes=24, seed=72, nonzero_bias=True)
    for g in (big, small):                                    # the second call has the smaller input and finds the first one's leftovers
        want, got, need = _both(X, g, compute, link=3)
        assert need <= X.XENOS_STATIC_WORKSPACE_BYTES
        assert np.isfinite(got).all()
        assert np.array_equal(want, got), g.name              # same kernels, same partitions: same bits


def test_static_workspace_rejects_plans_that_do_not_fit():
    X = _xenos()
    g = wg.vgg16(batch=8, hw=224, width=1.0, fc_dim=64, classes=8, seed=73, draw=False)
    s = X.Session(g, link=2, compute=1)
    try:
        assert s.info["workspace_bytes"] > X.XENOS_STATIC_WORKSPACE_BYTES
        with pytest.raises(X.XenosError) as ei:
            s.run_static()
        assert ei.value.status == X.XENOS_EUNSUPPORTED
        s.run()                                               # the plan itself is fine
        s.torch.cuda.synchronize()
    finally:
        s.close()
