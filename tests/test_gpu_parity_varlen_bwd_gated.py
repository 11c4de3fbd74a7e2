"""GPU parity of the gated backward pass over a packed variable-length batch (rodimus_chunk_scan_varlen_bwd_gated, with and
without the device-side cut) against the fp64 oracle ``scan_gated_bwd`` run on every sequence separately (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, rel_err, to_dev

pytestmark = pytest.mark.gpu

TOKEN_NAMES = ("dq", "dk", "dv", "dz_g", "dz_tau", "dz_beta")


@pytest.mark.parametrize("lengths,H,dv,cut,with_beta", [
    ([37, 1, 0, 130, 16, 65], 2, 128, False, True),      # ragged, single-token and empty sequences
    ([200, 33], 2, 256, False, False),                   # no value gate
    ([1500, 0, 700, 77], 2, 256, True, True),            # cut into segments of 256 tokens by the kernels
    ([512, 256, 257], 1, 128, True, True),
])
def test_matches_the_oracle_per_sequence(lengths, H, dv, cut, with_beta):
    print(f"varlen gated bwd {lengths} H{H} dv{dv} cut={cut} z_beta={with_beta}", flush=True)
    total, N = sum(lengths), len(lengths)
    d = wl.make_gated_scan_inputs(1, total, H, 64, dv, "bf16", s0_std=0.0, seed=total + dv)
    d = {k: (None if v is None else v[0]) for k, v in d.items()}
    if not with_beta:
        d["z_beta"] = None
    rng = np.random.Generator(np.random.PCG64(5))
    S0 = torch.from_numpy(rng.standard_normal((N, H, 64, dv), dtype=np.float32) * np.float32(0.1))
    d_o = torch.from_numpy(rng.standard_normal((total, H, dv), dtype=np.float32)).to(torch.bfloat16)
    dS_T = torch.from_numpy(rng.standard_normal((N, H, 64, dv), dtype=np.float32) * np.float32(0.1))
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lengths)]), dtype=torch.int32)
    g = to_dev(d)
    out = rodimus.rodimus_chunk_scan_varlen_bwd_gated(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], g["z_beta"], cu.cuda(), S0.cuda(),
                                                      d_o.cuda(), dS_T.cuda(), cut=cut)
    torch.cuda.synchronize()
    start = 0
    for b, n in enumerate(lengths):
        sl = slice(start, start + n)
        one = lambda x: None if x is None else x[sl][None]
        ref = oracle.scan_gated_bwd(one(d["q"]), one(d["k"]), one(d["v"]), one(d["z_g"]), one(d["z_tau"]), one(d["z_beta"]),
                                    S0[b][None], one(d_o), dS_T[b][None])
        if n > 0:
            for name in TOKEN_NAMES:
                if ref[name] is None:
                    assert out[name] is None
                    continue
                assert rel_err(out[name][sl][None], ref[name]) <= TOL_BF16, (b, n, name)
        assert rel_err(out["dS0"][b][None], ref["dS0"]) <= TOL_BF16, (b, n, "dS0")
        start += n
