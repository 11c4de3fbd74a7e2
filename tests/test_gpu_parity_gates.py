"""GPU parity of the DDTS gate front-end against the fp64 CPU oracle, alone and chained into the scan and the
decode step (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, TOL_F32, rel_err, to_dev

pytestmark = pytest.mark.gpu


def _check_gates(d, io):
    g = to_dev(d)
    la, beta, qo, ko = rodimus.rodimus_ddts_gates(g["z_g"], g["z_tau"], g.get("z_beta"), g["q"], g["k"])
    torch.cuda.synchronize()
    la_r, beta_r, qo_r, ko_r = oracle.ddts_gates(d["z_g"], d["z_tau"], d.get("z_beta"), d["q"], d["k"])
    tol_io = TOL_BF16 if io == "bf16" else TOL_F32
    assert rel_err(la, la_r) <= TOL_F32, "log_alpha"          # fp32 output of fp32 arithmetic
    if beta_r is not None:
        assert rel_err(beta, beta_r) <= TOL_F32, "beta"
    assert rel_err(qo, qo_r) <= tol_io and rel_err(ko, ko_r) <= tol_io
    # element by element as well (a relative bar on every entry that is not tiny)
    got, ref = la.double().cpu().numpy(), la_r
    assert np.all(np.abs(got - ref) <= 1e-5 * np.maximum(1.0, np.abs(ref)))
    return la, beta, qo, ko


@pytest.mark.parametrize("lead,dk,dv,io", [
    ((2, 100, 4), 64, 256, "bf16"),       # layer shape, odd row count per wavefront
    ((3, 7), 64, 128, "f32"),
    ((5,), 8, 8, "f32"),                  # one lane per row
    ((33,), 128, 40, "bf16"),
    ((3,), 512, 16, "f32"),               # a whole wavefront per row
])
def test_gates_match_the_oracle(lead, dk, dv, io):
    print(f"gates {lead} dk{dk} dv{dv} {io}", flush=True)
    d = wl.make_ddts_preactivations(lead, dk, dv, io, seed=dk + dv)
    _check_gates(d, io)


def test_gates_extreme_preactivations_zero_keys_and_in_place():
    d = wl.make_ddts_preactivations((6, 4), 64, 64, "f32", seed=3)
    d["z_g"][0] = -100.0        # g underflows, alpha = 1, alpha_hat -> 0
    d["z_g"][1] = 100.0         # g = 100: alpha = exp(-100 tau)
    d["z_tau"][2] = -100.0      # tau -> 0: alpha -> 1, alpha_hat -> 1
    d["z_tau"][3] = 100.0       # tau = 1
    d["z_g"][4, 0] = -104.0
    d["z_tau"][4, 0] = -104.0   # both degenerate: g^tau -> 1
    d["k"][5, 1] = 0.0          # zero key row stays zero
    la, beta, qo, ko = _check_gates(d, "f32")
    for t in (la, beta, qo, ko):
        assert torch.isfinite(t).all()
    assert (ko[5, 1] == 0).all()
    # in place: q_out = q, k_out = k
    g = to_dev(d)
    _, _, q2, k2 = rodimus.rodimus_ddts_gates(g["z_g"], g["z_tau"], None, g["q"], g["k"], q_out=g["q"], k_out=g["k"])
    torch.cuda.synchronize()
    assert q2.data_ptr() == g["q"].data_ptr() and torch.equal(q2, qo) and torch.equal(k2, ko)


def test_gates_then_scan_and_decode():
    """The whole DDTS path on the GPU: gate front-end -> chunk scan (MFMA path) -> decode step continuing from S_T,
    against the oracle's gate front-end feeding the oracle's recurrence."""
    B, T, H, dk, dv = 2, 321, 2, 64, 128
    d = wl.make_ddts_preactivations((B, T + 1, H), dk, dv, "bf16", seed=11)
    v = torch.from_numpy(np.random.default_rng(5).standard_normal((B, T + 1, H, dv)).astype(np.float32)).to(torch.bfloat16)
    g = to_dev(d)
    la, beta, qo, ko = rodimus.rodimus_ddts_gates(g["z_g"], g["z_tau"], g["z_beta"], g["q"], g["k"])
    vd = v.cuda()
    sl = lambda x: x[:, :T].contiguous()
    o, S_T = rodimus.rodimus_chunk_scan_fwd(sl(qo), sl(ko), sl(vd), sl(la), sl(beta), None, chunk=64)
    last = lambda x: x[:, T].contiguous()
    o_last = rodimus.rodimus_decode_step(last(qo), last(ko), last(vd), last(la), last(beta), S_T)
    torch.cuda.synchronize()
    # oracle chain in fp64 from the same pre-activations (its own gates, no rounding in between)
    la_r, beta_r, qo_r, ko_r = oracle.ddts_gates(d["z_g"], d["z_tau"], d["z_beta"], d["q"], d["k"])
    f32 = lambda x: x.astype(np.float32)
    o_r, S_r = oracle.scan(f32(qo_r), f32(ko_r), v, f32(la_r), f32(beta_r))
    assert rel_err(o, o_r[:, :T]) <= TOL_BF16
    assert rel_err(o_last, o_r[:, T]) <= TOL_BF16
    assert rel_err(S_T, S_r) <= TOL_BF16
