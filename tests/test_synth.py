"""The seeded input generator: reproducible, and bit-identical on the CPU and the GPU."""
import numpy as np
import pytest
import torch

from paper_2601_18383_amd import configs, synth


def test_streams_are_reproducible_and_distinct():
    wl = configs.get("cfg1")
    a, b = synth.Synth(wl), synth.Synth(wl)
    steps = torch.arange(1, 9)
    assert torch.equal(a.q(0, steps), b.q(0, steps))
    ka, va = a.kv(0, steps)
    assert not torch.equal(ka, va)
    # a step's tensors do not depend on which other steps are asked for
    assert torch.equal(a.q(0, torch.arange(5, 6))[0], a.q(0, steps)[4])
    # another seed, another stream
    import dataclasses
    c = synth.Synth(dataclasses.replace(wl, seed=wl.seed + 1))
    assert not torch.equal(c.q(0, steps), a.q(0, steps))


def test_value_distribution_and_planting():
    wl = configs.get("cfg3")
    g = synth.Synth(wl)
    steps = torch.arange(1, 65)
    k, v = g.kv(0, steps)
    assert abs(float(v.float().mean())) < 0.01 and abs(float(v.float().std()) - 1.0) < 0.02
    crit = g.critical(0, torch.arange(1, 4097))
    assert abs(float(crit.float().mean()) - 0.02) < 0.004
    mu = g.mean_query(0)
    assert torch.allclose(mu.norm(dim=-1), torch.full((wl.n_kv_heads,), wl.head_dim ** 0.25), atol=1e-4)
    # a planted key is 4 * mu on every KV head
    t, b = [int(x) for x in crit.nonzero()[0]]
    kk, _ = g.kv(0, torch.tensor([t + 1]))
    assert torch.equal(kk[0, b], (4.0 * mu).to(torch.bfloat16))
    lengths = g.decode_lengths()
    assert int(lengths.min()) >= 4096 and int(lengths.max()) <= 32768 and len(set(lengths.tolist())) > 20


def test_student_t_keys_are_heavy_tailed():
    g = synth.Synth(configs.get("cfg5"))
    k, _ = g.kv(0, torch.arange(1, 33))
    kf = k.float()
    assert float(kf.abs().max()) > 20.0 and abs(float(kf.median())) < 0.05
    s = synth.Synth(configs.get("cfg5b")).external_scores(torch.arange(1, 200))
    assert set(np.unique(s.numpy())) <= set(float(i) for i in range(64))


@pytest.mark.gpu
def test_cpu_and_gpu_generators_agree_bit_for_bit():
    for name in ("cfg1", "cfg5"):
        wl = configs.get(name)
        c, d = synth.Synth(wl, "cpu"), synth.Synth(wl, "cuda:0")
        steps = torch.arange(-3, 5)
        for layer in (0, wl.n_layers - 1):
            assert torch.equal(c.q(layer, steps), d.q(layer, steps).cpu())
            kc, vc = c.kv(layer, steps)
            kd, vd = d.kv(layer, steps)
            assert torch.equal(kc, kd.cpu()) and torch.equal(vc, vd.cpu())
    wl = configs.get("cfg1")
    sc, sd = synth.Synth(wl, "cpu").steady_state(0, 200), synth.Synth(wl, "cuda:0").steady_state(0, 200)
    for key in sc:
        assert torch.equal(sc[key], sd[key].cpu()), key
