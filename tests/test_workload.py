"""The seeded input generator: reproducible, sliceable, and of the stated distributions (no GPU)."""
import math

import torch

from paper_2411_00853_amd import workload as wl


def test_streams_are_reproducible_and_sliceable():
    r = wl.Rng(123, "cpu")
    a = r.normal(5, (1000,), 0.02)
    b = wl.Rng(123, "cpu").normal(5, (1000,), 0.02)
    assert torch.equal(a, b)
    assert torch.equal(r.normal(5, (100,), 0.02, offset=300), a[300:400])
    assert not torch.equal(r.normal(6, (1000,), 0.02), a)
    assert not torch.equal(wl.Rng(124, "cpu").normal(5, (1000,), 0.02), a)


def test_splitmix_reference_value():
    # splitmix64 with state 0: the first output of the published generator is 0xE220A8397B1DCDAF
    z = wl.hash64(0, torch.tensor([1], dtype=torch.int64))
    assert (int(z[0]) & ((1 << 64) - 1)) == 0xE220A8397B1DCDAF


def test_distributions():
    r = wl.Rng(9, "cpu")
    u = r.uniform(1, (200000,))
    assert 0.0 <= u.min() and u.max() < 1.0 and abs(u.mean().item() - 0.5) < 5e-3
    n = r.normal(2, (200000,), 0.02)
    assert abs(n.mean().item()) < 2e-4 and abs(n.std().item() - 0.02) < 2e-4
    k = 1 + r.binomial(3, (20000,), 9, 1.0 / 3.0)
    assert k.min() >= 1 and k.max() <= 10 and abs(k.float().mean().item() - 4.0) < 0.05
    t = r.randint(4, (100000,), 32000)
    assert t.min() >= 0 and t.max() < 32000 and t.max() > 31900


def test_gumbel_picks_follow_softmax():
    r = wl.Rng(11, "cpu")
    logits = torch.tensor([0.0, math.log(2.0), math.log(5.0)]).repeat(60000, 1)
    t = wl.pick_tokens(r, logits, 1.0, 77)
    f = torch.bincount(t.long(), minlength=3).double() / 60000
    assert (f - torch.tensor([1 / 8, 2 / 8, 5 / 8])).abs().max() < 0.01


def test_named_workloads_have_the_stated_shapes():
    w = wl.workload_7b()
    assert w.rows == 48 and w.shape.weight_elems() * 2 > 13.0e9
    d = wl.workload_dyn()
    assert d.batch == 32 and all(1 <= k <= 10 for k in d.lookahead) and all(512 <= n <= 4096 for n in d.kv_lens)
    assert d.rows <= 352 and max(n + k + 1 for n, k in zip(d.kv_lens, d.lookahead)) <= d.max_kv_len
    s = wl.make_stress(batch=2, K=2, vocab=500)
    assert s.target_logits.shape == (6, 500) and s.draft_logits.shape == (2, 2, 500)
    # the rank profile: sorted target logits fall like -1.1 ln(rank) (+ noise)
    top = torch.sort(s.target_logits[0], descending=True).values
    assert top[0] - top[249] > 1.1 * math.log(250) - 2.0
