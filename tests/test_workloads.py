"""The seeded input generators: shapes, counts, reproducibility.  CPU only; no method arithmetic here."""
import numpy as np
import torch

from paper_2502_11034_amd import workloads as W


def test_named_lists_have_the_stated_sizes():
    assert (len(W.tiny_transformer_list()), sum(s.numel for s in W.tiny_transformer_list())) == (27, 527872)
    assert (len(W.gpt2_small_list()), sum(s.numel for s in W.gpt2_small_list())) == (148, 124439808)
    specs = W.llama3_8b_list()
    assert (len(specs), sum(s.numel for s in specs)) == (291, 8030261248)
    assert len(specs) == 9 * 32 + 3                      # 9 tensors per dense decoder layer + 3 (Sec. 4.3)
    assert max(s.numel for s in specs) == 128256 * 4096
    per_layer = sum(s.numel for s in specs if s.name.startswith("l0."))
    assert per_layer == 218112000
    ragged = W.ragged_stress_list()
    sizes = np.array([s.numel for s in ragged[:-1]])
    assert len(ragged) == 20001 and sizes.min() >= 1 and sizes.max() <= 4194304
    assert ragged[-1].numel == 128256 * 4096
    # log-uniform: about a third of the sizes in each third of the log range
    thirds = np.histogram(np.log(sizes), bins=3, range=(0, np.log(4194304)))[0] / len(sizes)
    assert (np.abs(thirds - 1 / 3) < 0.02).all()


def test_gradients_are_reproducible_per_tensor_and_step():
    w = W.config1()
    a = w.make_grad(5, 3, "cpu")
    b = w.make_grad(5, 3, "cpu")
    c = w.make_grad(5, 4, "cpu")
    d = w.make_grad(6, 3, "cpu")
    assert torch.equal(a, b) and not torch.equal(a, c) and a.shape != d.shape or not torch.equal(a[:8], d[:8])
    assert a.dtype == torch.float32 and a.numel() == w.numels[5]
    sig = float(a.double().std())
    assert 0.5 * w.sigma[5] < sig < 2.0 * w.sigma[5]
    assert 1e-4 <= w.sigma.min() and w.sigma.max() <= 1e-1


def test_spike_schedules():
    w1 = W.config1()
    assert sorted(w1.spikes) == [7, 13] and all(len(idx) == 3 and f == 100.0 for idx, f in w1.spikes.values())
    i = int(w1.spikes[7][0][0])
    assert w1.grad_scale(i, 7) == 100.0 * w1.grad_scale(i, 6)
    w2 = W.config2()
    assert 4 in w2.spikes and len(w2.spikes[4][0]) == 7 and w2.spikes[4][1] == 50.0       # 5 % of 148
    w3 = W.config3()
    assert 3 in w3.spikes and len(w3.spikes[3][0]) == 15 and w3.bf16_copy
    w4 = W.config4()
    assert w4.grad_dtype == torch.bfloat16 and w4.bf16_copy


def test_heavy_tail_outliers_and_state_init():
    w = W.config5(W.ragged_stress_list(3, 1 << 18, None, seed=3) + [W.TensorSpec("big", (400000,), "matrix")])
    g = w.make_grad(3, 1, "cpu")
    z = (g / float(w.sigma[3])).abs()
    # ~400 elements are replaced by sigma*t(nu=2); P(|t2| > 6) = 1 - 6/sqrt(38) = 2.7 % of those, and a
    # Gaussian puts nothing beyond 6 sigma in 400 000 draws
    assert 3 <= int((z > 6).sum()) <= 30
    plain = W.Workload(w.specs).make_grad(3, 1, "cpu")
    assert int(((plain / float(w.sigma[3])).abs() > 6).sum()) == 0
    specs = [W.TensorSpec("w", (64, 8), "matrix"), W.TensorSpec("n", (8,), "norm"), W.TensorSpec("b", (8,), "bias")]
    wl = W.Workload(specs, bf16_copy=True)
    p, m, v, c = wl.make_state("cpu")
    assert float(p[1].min()) == 1.0 and float(p[2].abs().max()) == 0.0 and 0.01 < float(p[0].std()) < 0.03
    assert all(float(x.abs().max()) == 0.0 for x in m + v)
    assert c[0].dtype == torch.bfloat16 and torch.equal(c[0], p[0].to(torch.bfloat16))
    p2, m2, v2, c2 = wl.make_state("cpu", "lion")
    assert v2 is None and torch.equal(p[0], p2[0])
    bits = W.to_numpy(c[1])
    assert bits.dtype == np.uint16 and (bits == 0x3F80).all()
