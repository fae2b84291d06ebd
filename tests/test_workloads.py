"""The synthetic workloads have the sizes the benchmark definition states and are seeded."""
import numpy as np
import torch

from paper_2506_16235_amd import workloads as W


def test_model_shapes():
    r = W.resnet50_sizes()
    assert len(r) == 161 and sum(r) == 25_557_032
    assert min(r) == 64 and max(r) == 2_359_296 and sum(1 for x in r if x <= 2048) == 107
    b = W.bert_base_sizes()
    assert len(b) == 199 and sum(b) == 109_482_240 and b[0] == 30522 * 768 == 23_440_896
    l = W.llama7b_sizes()
    assert len(l) == 291 and sum(l) == 6_738_415_616
    off = W.llama7b_bucket_offsets()
    assert len(off) - 1 == 258 and int(off[-1]) == 6_738_415_616
    assert int(off[1]) == 26_214_400 and int(off[-1] - off[-2]) == 1_314_816


def test_generators_are_seeded_and_shaped():
    g1, off1 = W.cfg1()
    g1b, _ = W.cfg1()
    assert g1.numel() == 1 << 20 and torch.equal(g1, g1b)
    assert abs(float(g1.std()) - 1e-3) < 2e-5
    a, off = W.resnet50_grad(3)
    b, _ = W.resnet50_grad(3)
    c, _ = W.resnet50_grad(4)
    assert torch.equal(a, b) and not torch.equal(a, c)
    sig = W.resnet50_sigmas()
    assert sig.min() >= 1e-5 and sig.max() <= 1e-2
    lo, hi = int(off[-3]), int(off[-2])                 # fc weight, 2,048,000 elements
    assert abs(float(a[lo:hi].std()) / sig[-2] - 1) < 0.01


def test_bert_embedding_sparsity():
    small = W.scaled_model_like(W.bert_base_sizes(), 64)
    assert len(small) == 199
    gen = W._gen("cpu", 1)
    x = W._laplace(200000, 1e-4, gen, "cpu")
    assert torch.isfinite(x).all()
    assert abs(float(x.abs().mean()) / 1e-4 - 1) < 0.02      # E|x| = b for Laplace(0, b)
    t = W._student_t3(200000, 1e-4, gen, "cpu")
    assert torch.isfinite(t).all() and float(t.abs().max()) > 1e-3   # heavy tails


def test_bandwidth_trace():
    bw = W.bandwidth_trace(200)
    assert len(bw) == 200 and bw.min() >= 1e9 and bw.max() <= 1e11
    assert np.array_equal(bw, W.bandwidth_trace(200))
    changes = np.count_nonzero(np.diff(bw))
    assert 5 <= changes <= 40
    assert W.simulated_tx_seconds(1.25e6, 1e9) == 0.010 + 0.010
