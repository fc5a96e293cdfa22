"""uniql_w4_mlp_static (the entry point that allocates nothing: its workspace is a static array in device memory)
against uniql_w4_mlp on a caller's workspace, through the C ABI: two calls in a row, the second with a smaller input."""
import ctypes as C

import numpy as np
import pytest

import workloads as wl
from workloads import Keep

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2512_03383_amd as uq
    uq.lib()
    torch.cuda.set_device(0)
    return uq, torch


def _call(uq, torch, fn_name, qws, keeps, x, workspace=None):
    """One call through the C ABI proper (ctypes on the library's exported symbol)."""
    L = uq.lib()
    Wd = (uq.W4 * 3)(*[w.desc() for w in qws])
    kd = (uq.KeepDesc * 3)(*[uq._keep_desc(k) or uq.KeepDesc() for k in keeps])
    n_out = uq.kept_dims(qws[2], keeps[2])[0]
    y = torch.full((n_out,), 7.0, dtype=torch.float16, device="cuda")
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if fn_name == "uniql_w4_mlp_static":
        rc = L.uniql_w4_mlp_static(Wd, kd, C.c_void_p(x.data_ptr()), C.c_void_p(y.data_ptr()), stream)
    else:
        rc = L.uniql_w4_mlp(Wd, kd, C.c_void_p(x.data_ptr()), C.c_void_p(y.data_ptr()),
                            C.c_void_p(workspace.data_ptr()), int(workspace.numel()), stream)
    assert rc == 0, uq.strerror(rc)
    torch.cuda.synchronize()
    return y


def test_static_workspace_matches_callers_workspace(env):
    uq, torch = env
    rng = wl.rng_for(17, 1)
    # the Llama-3-8B shaped MLP (the single persistent launch), first at 15 %, then at 35 % (a smaller input:
    # fewer intermediate channels, so part of what the first call left in the array stays behind)
    ws = [wl.gen_linear(rng, 14336, 4096), wl.gen_linear(rng, 14336, 4096), wl.gen_linear(rng, 4096, 14336)]
    qws = [uq.QuantLinear.from_numpy(w) for w in ws]
    work = uq.mlp_workspace(14336)
    x = torch.from_numpy(wl.gen_activations(rng, 1, 4096)[0]).cuda()
    for n_hidden in (12185, 9318):
        keeps = [Keep(n_keep=n_hidden), Keep(n_keep=n_hidden), Keep(k_keep=n_hidden)]
        y_static = _call(uq, torch, "uniql_w4_mlp_static", qws, keeps, x)
        y_work = _call(uq, torch, "uniql_w4_mlp", qws, keeps, x, work)
        assert torch.isfinite(y_static).all()
        assert torch.equal(y_static, y_work), n_hidden       # integer-exact bar: the same kernels on the same inputs
    # ... then a shape that runs as two launches through the array (1700 of 2048 intermediate channels)
    ws = [wl.gen_linear(rng, 2048, 1024), wl.gen_linear(rng, 2048, 1024), wl.gen_linear(rng, 1024, 2048)]
    qws = [uq.QuantLinear.from_numpy(w) for w in ws]
    x = torch.from_numpy(wl.gen_activations(rng, 1, 1024)[0]).cuda()
    for n_hidden in (1700, 900):
        keeps = [Keep(n_keep=n_hidden), Keep(n_keep=n_hidden), Keep(k_keep=n_hidden)]
        assert torch.equal(_call(uq, torch, "uniql_w4_mlp_static", qws, keeps, x),
                           _call(uq, torch, "uniql_w4_mlp", qws, keeps, x, uq.mlp_workspace(2048)))


def test_static_workspace_refuses_what_does_not_fit(env):
    uq, torch = env
    L = uq.lib()
    assert L.uniql_w4_mlp_static_max_hidden() == 32768
    rng = wl.rng_for(17, 2)
    big = uq.QuantLinear.from_numpy(wl.gen_linear(rng, 32768 + 128, 128))     # 32896 intermediate channels
    down = uq.QuantLinear.from_numpy(wl.gen_linear(rng, 128, 32768 + 128))
    x = torch.zeros(128, dtype=torch.float16, device="cuda")
    y = torch.zeros(128, dtype=torch.float16, device="cuda")
    Wd = (uq.W4 * 3)(big.desc(), big.desc(), down.desc())
    rc = L.uniql_w4_mlp_static(Wd, None, C.c_void_p(x.data_ptr()), C.c_void_p(y.data_ptr()), None)
    assert rc == uq.UNIQL_E_SHAPE, uq.strerror(rc)
