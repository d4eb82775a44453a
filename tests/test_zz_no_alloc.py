"""The accept / resample entry point that allocates nothing (seed_accept_resample_static: row statistics in an
array of the library's device image) against the stand-alone entry point, through the C ABI: two calls in a row
on one stream, the second with a smaller input, so that whatever the first call left in the array is there
when the second runs."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from workloads.device import f32, i32

pytestmark = pytest.mark.gpu


def _case(seed, N, G, Tp, V, temp):
    rng = np.random.default_rng(seed)
    logits = (rng.standard_normal((N, Tp, V)) * 2.0).astype(np.float32)
    q = oracle.softmax_temperature(logits[:, :G] + (rng.standard_normal((N, G, V)) * 0.5).astype(np.float32), temp)
    u = wl.uniform24(seed, (2, N, G))
    return logits, q, wl.draw_tokens(q, u[0]), u[1], wl.uniform24(seed + 1, (N,))


def _both(sv, logits, q, drafts, u_acc, u_res, **kw):
    a = [f32(logits), None if q is None else f32(q), i32(drafts), None if u_acc is None else f32(u_acc),
         None if u_res is None else f32(u_res)]
    N, G = drafts.shape
    outs = sv.binding._accept_outputs(N, G, "cuda:0")           # preallocated: the call itself allocates nothing
    for o in outs:
        o.fill_(-7)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    got = sv.accept_resample(*a, static_scratch=True, outs=outs, **kw)
    assert torch.cuda.memory_allocated() == before
    want = sv.accept_resample(*a, **kw)
    torch.cuda.synchronize()
    return [g.cpu().numpy() for g in got], [w.cpu().numpy() for w in want]


def test_static_scratch_entry_point_matches_the_standalone_one():
    import paper_2406_18200_amd as sv
    # first a large call (96 target rows: four statistics slices per row), then a smaller one (12 rows, sixteen
    # slices per row: a different layout over the same array), then greedy mode, then the bonus-row form
    for seed, N, G, Tp, V, temp, greedy in ((1, 16, 6, 6, 32000, 1.0, False), (2, 3, 4, 4, 32000, 0.7, False),
                                            (3, 5, 3, 3, 1024, 1.0, True), (4, 2, 2, 3, 517, 0.9, False)):
        print(f"case N={N} G={G} Tp={Tp} V={V} greedy={greedy}", flush=True)
        logits, q, drafts, u_acc, u_res = _case(seed, N, G, Tp, V, temp)
        if greedy:
            got, want = _both(sv, logits, None, drafts, None, None, kind="logits", greedy=True)
        else:
            got, want = _both(sv, logits, q, drafts, u_acc, u_res, kind="logits", temperature=temp)
        # integer outputs bit for bit; p(x) to the last bits (the statistics are summed in a different order)
        for g, w_, name in zip(got[:3], want[:3], ("accept_len", "out_tok", "n_out")):
            assert np.array_equal(g, w_), name
        assert np.allclose(got[3], want[3], rtol=2e-6, atol=0)
        # and against the oracle's decisions (no near-ties for these seeds)
        if not greedy:
            ref = oracle.accept_resample(oracle.softmax_temperature(logits, temp), q, drafts, u_acc, u_res)
        else:
            ref = oracle.accept_resample(None, None, drafts, None, None, greedy=True, logits=logits)
        assert np.array_equal(got[0], ref[0]) and np.array_equal(got[2], ref[2])
    # the PROBS kind needs no statistics and is bit-exact against the oracle
    rng = np.random.default_rng(9)
    p = oracle.softmax_temperature(rng.standard_normal((4, 3, 300)) * 2, 1.0)
    qq = oracle.softmax_temperature(rng.standard_normal((4, 3, 300)) * 2, 1.0)
    u = wl.uniform24(9, (2, 4, 3))
    d = wl.draw_tokens(qq, u[0])
    ur = wl.uniform24(10, (4,))
    got = sv.accept_resample(f32(p), f32(qq), i32(d), f32(u[1]), f32(ur), kind="probs", static_scratch=True)
    for g, w_ in zip(got, oracle.accept_resample(p, qq, d, u[1], ur)):
        assert np.array_equal(g.cpu().numpy(), w_)


def test_static_scratch_entry_point_rejects_too_many_rows():
    import paper_2406_18200_amd as sv
    N, G, V = 1025, 4, 16                                  # 4100 target rows > 4096
    z = torch.zeros((N, G, V), device="cuda")
    with pytest.raises(sv.SeedError) as e:
        sv.accept_resample(z, z, torch.zeros((N, G), dtype=torch.int32, device="cuda"), torch.zeros((N, G), device="cuda"),
                           torch.zeros(N, device="cuda"), kind="logits", static_scratch=True)
    assert e.value.code == -3
