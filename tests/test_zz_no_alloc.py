"""quamba_mixer_decode_noalloc (the generation step for callers that cannot allocate: its scratch is a
buffer built into the library) against quamba_mixer_decode with a caller workspace: the same kernels on
another scratch address, so outputs and carried states must be the same bits.  Two calls in a row share
the built-in buffer, the second with a smaller batch (what the first left behind must not matter)."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2410_13229_amd as Q
import workloads as W
from gpu_util import dev, empty, host, oracle_setup, qweights_to_dev, rel_err, workspace

pytestmark = pytest.mark.gpu


def _step(cfg, qd, sc, Bt, stream_id, noalloc):
    ssm_np, cs_np = W.make_decode_state(cfg, batch=Bt)
    ssm, cs = dev(ssm_np), dev(cs_np)
    u = W.make_hidden(cfg, batch=Bt, seqlen=1, stream=stream_id)
    out = torch.zeros((Bt, cfg.d_model), dtype=torch.float16, device="cuda:0")
    if noalloc:
        Q.quamba_mixer_decode_noalloc(cfg, qd, sc, dev(u[:, 0]), Bt, out, ssm, cs, None)
    else:
        ws = workspace(Q.quamba_workspace_bytes(cfg, Bt, 1))
        Q.quamba_mixer_decode(cfg, qd, sc, dev(u[:, 0]), Bt, out, ssm, cs, None, ws)
    return host(out), host(ssm), host(cs), (u, ssm_np, cs_np)


def test_decode_noalloc_matches_decode_on_two_calls_in_a_row():
    cfg = W.CONFIGS["c2"]
    w, qw, sc = oracle_setup(cfg)
    qd = qweights_to_dev(qw)
    assert Q.quamba_workspace_bytes(cfg, 64, 1) <= 48 << 20
    for Bt, sid in ((64, 500), (5, 501)):  # the second call is smaller and finds the first call's leftovers
        a = _step(cfg, qd, sc, Bt, sid, noalloc=True)
        b = _step(cfg, qd, sc, Bt, sid, noalloc=False)
        assert np.array_equal(a[0].view(np.uint16), b[0].view(np.uint16)), Bt
        assert np.array_equal(a[1].view(np.uint32), b[1].view(np.uint32)), Bt
        assert np.array_equal(a[2].view(np.uint16), b[2].view(np.uint16)), Bt
        u, ssm_np, cs_np = a[3]
        ref = O.q_decode(qw, sc, u[:, 0], ssm_np, cs_np)
        assert rel_err(a[0].astype(np.float64), ref["out"][:, 0].astype(np.float64)) <= 2e-2
        assert rel_err(a[1], ref["h"]) <= 1e-3
        assert np.array_equal(a[2].view(np.uint16), ref["conv_state"].view(np.uint16))


def test_decode_noalloc_rejects_what_does_not_fit():
    cfg = W.CONFIGS["c2"]
    w, qw, sc = oracle_setup(cfg)
    qd = qweights_to_dev(qw)
    Bt = 256  # beyond the built-in buffer at this width
    assert Q.quamba_workspace_bytes(cfg, Bt, 1) > 48 << 20
    z = torch.zeros((Bt, cfg.d_model), dtype=torch.float16, device="cuda:0")
    ssm = torch.zeros((Bt, cfg.d_inner, 16), dtype=torch.float32, device="cuda:0")
    cs = torch.zeros((Bt, cfg.d_inner, 3), dtype=torch.float16, device="cuda:0")
    with pytest.raises(Q.QuambaError) as e:
        Q.quamba_mixer_decode_noalloc(cfg, qd, sc, z, Bt, z.clone(), ssm, cs, None)
    assert e.value.code == -3 and "scratch" in str(e.value)
