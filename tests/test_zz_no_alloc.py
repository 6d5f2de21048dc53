"""ep_layout_static, the entry point that allocates nothing (scratch in a static device array), against
ep_layout, the entry point it is a variant of, through the C ABI: every output array bit for bit, on two
calls in a row, the second with a smaller input; then the oracle as a second opinion."""
import numpy as np
import pytest

import ep_inputs as g

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

NAMES = ("count", "expert_total", "rank_total", "base", "expert_offset", "rank_offset", "slot", "dst_row")


def _outputs(S, T, K, E, R):
    i32 = dict(dtype=torch.int32, device="cuda")
    shapes = dict(count=(S, E), expert_total=(E,), rank_total=(R,), base=(S, E), expert_offset=(E + 1,),
                  rank_offset=(R + 1,), slot=(S, T, K), dst_row=(S, T, K))
    return {n: torch.full(shapes[n], -7, **i32) for n in NAMES}


@pytest.mark.parametrize("cid,T2", [(4, 1000), (2, 37), (5, 8191), (1, 5)])
def test_layout_static_equals_layout_on_two_calls_in_a_row(oracle, cid, T2):
    import paper_2512_19849_amd as ep
    from paper_2512_19849_amd.runner import EPRunner
    ep.load_library(build_if_missing=False)
    cfg = g.config(cid)
    S, K, E, R = cfg.S, cfg.K, cfg.E, cfg.R
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    with EPRunner(R, E, K, cfg.H, cfg.T, S=S, num_proxy_threads=0) as r:
        for T in (cfg.T, T2):                                   # the second call is the smaller one
            idx, _ = g.routing_all(cfg, T)
            if T == T2:
                idx = g.mask_random(idx, 0.1, seed=5)
            d_idx = torch.from_numpy(idx).cuda()
            got = _outputs(S, T, K, E, R)
            ep.ep_layout_static(d_idx, S, T, K, E, R, *(got[n] for n in NAMES), status)
            ref = r.layout(d_idx).numpy()
            torch.cuda.synchronize()
            want = oracle.layout(idx, E, R)
            for n in NAMES:
                assert np.array_equal(got[n].cpu().numpy(), ref[n]), (n, T, "vs ep_layout")
                assert np.array_equal(ref[n], want[n]), (n, T, "vs oracle")
    assert int(status.item()) == 0


def test_layout_static_limits_and_status_word():
    import paper_2512_19849_amd as ep
    ep.load_library(build_if_missing=False)
    S, T, K, E, R = 1, 100, 2, 8, 2
    rng = np.random.default_rng(1)
    idx = np.stack([rng.permutation(E)[:K] for _ in range(T)]).astype(np.int32)[None]
    idx[0, 41, 1] = E                                           # out of range: reported, entry dropped
    d_idx = torch.from_numpy(idx).cuda()
    got = _outputs(S, T, K, E, R)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    ep.ep_layout_static(d_idx, S, T, K, E, R, *(got[n] for n in NAMES), status)
    torch.cuda.synchronize()
    assert int(status.item()) == ep.EP_EBOUNDS
    assert got["slot"][0, 41, 1].item() == -1 and got["dst_row"][0, 41, 1].item() == -1
    assert int(got["expert_total"].sum().item()) == T * K - 1
    ep.ep_layout_static(d_idx, S, T, K, E, R, *(got[n] for n in NAMES), None)      # no status word: still runs
    torch.cuda.synchronize()
    # beyond the static buffer: (S * ceil(T/64) + 1) * E > 262144
    S2, T2, E2 = 4, 64 * 70, 1024
    big = torch.zeros((S2, T2, 1), dtype=torch.int32, device="cuda")
    out = _outputs(S2, T2, 1, E2, 1)
    with pytest.raises(ep.EPError) as ei:
        ep.ep_layout_static(big, S2, T2, 1, E2, 1, *(out[n] for n in NAMES), None)
    assert ei.value.rc == ep.EP_EINVAL
    assert "static buffer holds 262144" in ep.ep_last_error()
    for bad in (dict(E=7, R=2), dict(K=0), dict(S=0), dict(T=-1), dict(R=0)):
        kw = dict(S=S, T=T, K=K, E=E, R=R)
        kw.update(bad)
        with pytest.raises(ep.EPError):
            ep.ep_layout_static(d_idx, kw["S"], kw["T"], kw["K"], kw["E"], kw["R"], *(got[n] for n in NAMES), None)
