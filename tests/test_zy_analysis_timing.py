"""A wall-clock check, kept apart from the parity tests and collected after them: the static
analyser's predicted step time against a measured one."""
import numpy as np
import pytest
import torch

import paper_2204_06514_amd as fax
from workloads.configs import ADAMW_DEFAULT
from helpers import DEV, dims_of
from test_gpu_train import _like

pytestmark = pytest.mark.gpu


def test_static_analysis_predicts_the_measured_step_time():
    """fax_analyze prices the step from the library's own launch plans; the prediction has to be
    in the neighbourhood of what the GPU then takes (a 2-layer cut of the 700M-parameter config).
    A sanity bound, not a performance claim: a factor of two either way, so that a slow or shared
    GPU does not fail it (measured ratios: 0.95-1.07)."""
    from workloads import get_config
    ms = get_config("cfg5").scaled(L=2)
    sh = ms.blk
    md = fax.FaxModelDims(dims_of(sh), sh.L, ms.V, ms.S_max, 0)
    predicted = fax.fax_analyze(md).ms_step
    rng = np.random.default_rng(0)
    mk = lambda *shape: (0.02 * torch.randn(*shape, device=DEV)).to(torch.bfloat16)
    Hd = sh.H * sh.dh
    blk = lambda: {"ln1_g": mk(sh.D) + 1, "ln1_b": mk(sh.D), "wqkv": mk(sh.D, 3 * Hd), "bqkv": mk(3 * Hd), "wo": mk(Hd, sh.D),
                   "bo": mk(sh.D), "ln2_g": mk(sh.D) + 1, "ln2_b": mk(sh.D), "w1": mk(sh.D, sh.F), "b1": mk(sh.F),
                   "w2": mk(sh.F, sh.D), "b2": mk(sh.D)}
    params = {"tok_emb": mk(ms.V, sh.D), "pos_emb": mk(ms.S_max, sh.D), "lnf_g": mk(sh.D) + 1, "lnf_b": mk(sh.D),
              "blocks": [blk() for _ in range(sh.L)]}
    master = _like(params, src=params); m = _like(params, 0.0); v = _like(params, 0.0); grads = _like(params, 0.0)
    tok = torch.from_numpy(rng.integers(0, ms.V, (sh.B, sh.S), dtype=np.int32)).to(DEV)
    lab = torch.from_numpy(rng.integers(0, ms.V, (sh.B, sh.S), dtype=np.int32)).to(DEV)
    wsb = fax.fax_train_workspace_bytes(md)
    ws = torch.empty(wsb, dtype=torch.uint8, device=DEV)
    loss = torch.zeros(4, device=DEV)
    hp = fax.FaxAdamW(**ADAMW_DEFAULT)
    tabs = [fax.model_tensors(t) for t in (params, master, m, v, grads)]
    step = lambda t: fax.fax_train_step(md, *tabs, tok, lab, hp, t, loss, ws, wsb)
    for t in (1, 2):
        step(t)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for t in (3, 4, 5, 6):
        step(t)
    e1.record()
    torch.cuda.synchronize()
    measured = e0.elapsed_time(e1) / 4
    assert np.isfinite(loss[0].item())
    assert 0.5 < predicted / measured < 2.0, (predicted, measured)
