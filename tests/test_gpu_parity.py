"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element, on
the same seeded inputs.  Sizes here span several tiles, ragged tails and unaligned bucket
starts while the oracle still finishes in seconds."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_16235_amd import binding as nsml
from paper_2506_16235_amd import workloads as W
from gpu_util import DEV, Case, say

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["auto", "dense"])
def path(request, monkeypatch):
    """Every case runs twice: with the paths the library picks itself (what the streaming pass
    stages comes from a sample of the gradient; buckets fall back to the dense passes on their
    own when they must), and with every bucket forced through the dense passes.  The switches
    are nsml_set_option settings applied to every context the test creates."""
    monkeypatch.setitem(nsml.Context.default_options, "force_dense", 1 if request.param == "dense" else 0)
    return request.param


def _rand(n, seed, sigma=1e-3):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    return torch.randn(n, generator=g, device=DEV) * sigma


def test_cfg1_single_vector(path):
    """Configuration 1: 1,048,576 x N(0, 1e-3), ratio 0.01 (k = 10,486), int8, chunk 2048."""
    g, off = W.cfg1(DEV)
    c = Case(g, off)
    K, vb, ns = c.step(0.01, 8)
    assert (K, vb, ns) == (10486, 10486, 6)
    assert c.ctx.path_stats() == ((0, 1) if path == "dense" else (1, 0))


@pytest.mark.parametrize("bits", [4, 8, 16, 32])
def test_ragged_unaligned_buckets(bits):
    """Bucket starts at every alignment mod 4, an empty bucket, 1-element buckets, a bucket that
    ends one element into a tile, several tiles per bucket."""
    sizes = [1, 64, 2048, 0, 4095, 4097, 3, 17889, 8192, 12289, 1, 50001, 7, 131072 + 5]
    off = W.offsets_of(sizes)
    n = int(off[-1])
    say("ragged", bits, n)
    c = Case(_rand(n, 100 + bits), off, chunk=64)
    for step, ratio in enumerate((0.3, 0.05, 0.002, 1.0)):
        c.set_grad(_rand(n, 200 + 10 * bits + step))
        c.step(ratio, bits)


@pytest.mark.parametrize("chunk", [8, 64, 256, 264, 2048, 4096])
@pytest.mark.parametrize("bits", [4, 8, 16])
def test_high_ratios_and_chunk_lengths(bits, chunk):
    """Ratios from an eighth up: the survivors are written and coded from the dense accumulator
    in one pass: a wavefront per chunk of up to 256 survivors, the workgroup per chunk of up to
    2048; longer chunks (4096) take the ordered write and a coding pass of their own.  Buckets from a
    few elements to many spans, unaligned starts, an empty one; the third step runs on the
    residual of the first two, the last one on a gradient with 70 % exact zeros."""
    sizes = [5, 70_000, 0, 1_000_003, 257, 4096, 300_001, 9, 2_500_000]
    off = W.offsets_of(sizes)
    n = int(off[-1])
    c = Case(_rand(n, 900 + bits + chunk), off, chunk=chunk)
    for step, ratio in enumerate((0.5, 0.2, 1.0, 0.13)):
        c.set_grad(_rand(n, 950 + 10 * step + bits))
        c.step(ratio, bits)
    g = _rand(n, 990 + bits)
    z = torch.rand(n, generator=torch.Generator(device=DEV).manual_seed(5), device=DEV)
    g[z < 0.7] = 0.0
    c.set_grad(g)
    c.set_residual(np.zeros(n, dtype=np.float32))
    c.step(0.45, bits)
    c.step(0.3, bits)


@pytest.mark.parametrize("ratio,bits", [(0.1, 8), (0.01, 4), (0.5, 32), (1.0, 32), (1.0, 4)])
def test_heavy_ties_and_zeros(ratio, bits):
    """Magnitudes drawn from a handful of values, 60 % exact zeros of both signs: the threshold
    sits inside a huge group of equal keys and ties must go to the lowest indices."""
    n = 300_000
    gen = torch.Generator(device=DEV)
    gen.manual_seed(7)
    lv = torch.randint(-3, 4, (n,), generator=gen, device=DEV).float() * 0.25
    z = torch.rand(n, generator=gen, device=DEV)
    lv[z < 0.6] = 0.0
    lv[z < 0.3] = -0.0
    off = W.offsets_of([100_000, 150_001, 49_999])
    c = Case(lv, off, chunk=256)
    c.step(ratio, bits)


def test_all_zero_and_constant_buckets():
    n = 40_000
    g = torch.zeros(n, device=DEV)
    g[10_000:20_000] = 3.0
    g[20_000:30_000] = -1e-30          # subnormal-scale products must not be flushed
    g[30_000:] = torch.arange(10_000, device=DEV).float() * 1e-42    # subnormals
    off = W.offsets_of([10_000] * 4)
    for bits in (8, 4, 16, 32):
        c = Case(g.clone(), off, chunk=8)
        c.step(0.01, bits)
        c.step(0.37, bits)             # residual carried


def test_identity_ratio1_bits32():
    n = 70_001
    g = _rand(n, 3)
    c = Case(g, W.offsets_of([n]))
    idx, val, sc = c.ctx.compress(c.g, c.r, c.off, 1.0, 32)
    assert torch.equal(idx.view(torch.int32), torch.arange(n, device=DEV, dtype=torch.int32))
    assert torch.equal(val[:4 * n].view(torch.float32), g)
    assert torch.count_nonzero(c.r) == 0
    d = c.ctx.decompress(idx, val, sc, n, c.off, 1.0, 32)
    assert torch.equal(d, g)


def test_error_feedback_conservation_on_gpu():
    """decompressed + new residual == grad + old residual, exactly, on the GPU's own outputs."""
    n = 500_000
    c = Case(_rand(n, 11), W.offsets_of([123_457, 376_543]))
    c.set_residual(_rand(n, 12).cpu().numpy())
    acc = c.g + c.r
    for bits in (4, 8, 16):
        r0 = c.r.clone()
        acc = c.g + r0
        idx, val, sc = c.ctx.compress(c.g, c.r, c.off, 0.02, bits)
        d = c.ctx.decompress(idx, val, sc, n, c.off, 0.02, bits)
        assert torch.equal(d + c.r, acc)


def test_resnet50_shaped_scaled_ef_steps():
    """Configuration 2 at 1/16 scale: 161 buckets (107 tiny), sigma_l per layer, ratio 0.05,
    int8, residual carried over 4 steps with a fresh gradient each step."""
    sizes = W.scaled_model_like(W.resnet50_sizes(), 16)
    off = W.offsets_of(sizes)
    sig = W.resnet50_sigmas()
    n = int(off[-1])
    c = None
    for step in range(4):
        g = torch.empty(n, device=DEV)
        for b, nb in enumerate(sizes):
            g[int(off[b]):int(off[b + 1])] = W._normal(nb, float(sig[b]), W._gen(DEV, W.make_seed(2, step, b)), DEV)
        if c is None:
            c = Case(g, off)
        else:
            c.set_grad(g)
        c.step(0.05, 8)


@pytest.mark.parametrize("bits", [4, 8, 32])
def test_clustered_survivors_overflow_staging_segments(path, bits):
    """Survivors packed into runs longer than a staging segment holds (an embedding whose few
    touched rows carry all the large values): those segments are read from the dense accumulator
    instead, and the bucket's survivors are then taken from there too; no dense passes.  Three
    steps, with the residual of the steps before."""
    n0, n1 = 1_500_000, 40_000
    gen = torch.Generator(device=DEV)
    gen.manual_seed(31 + bits)
    g = W._laplace(n0 + n1, 1e-6, gen, DEV)
    for start in range(10_000, n0 - 5_000, 60_000):
        g[start:start + 3_000] = W._laplace(3_000, 1e-3, gen, DEV)
    off = np.array([0, n0, n0 + n1], dtype=np.uint64)
    c = Case(g, off, chunk=256)
    for step, ratio in enumerate((0.04, 0.05, 0.02)):
        c.step(ratio, bits)
        st = c.ctx.bucket_state(0)
        say("clustered", bits, path, ratio, st)
        if path == "auto":
            assert st["path"] == 2, st               # threshold from staged + dense segments, survivors from the accumulator
        g2 = W._laplace(n0 + n1, 1e-6, gen, DEV)
        for start in range(10_000 + 777 * (step + 1), n0 - 5_000, 60_000):
            g2[start:start + 3_000] = W._laplace(3_000, 1e-3, gen, DEV)
        c.set_grad(g2)


@pytest.mark.parametrize("ratio", [0.1, 0.05, 0.01, 0.001])
@pytest.mark.parametrize("bits", [8, 4])
def test_bert_shaped_scaled(ratio, bits):
    """Configuration 3 at 1/24 scale in every tensor but with the embedding's structure kept:
    95 % of its rows exactly zero, so at ratio 0.1 the cut falls among the zeros."""
    sizes = W.scaled_model_like(W.bert_base_sizes(), 24)
    rows = 30522 // 24
    sizes[0] = rows * 768
    off = W.offsets_of(sizes)
    n = int(off[-1])
    g = torch.empty(n, device=DEV)
    for b, nb in enumerate(sizes):
        gen = W._gen(DEV, W.make_seed(3, 0, b))
        if b == 0:
            emb = g[:nb].view(rows, 768)
            emb.zero_()
            nz = torch.randperm(rows, generator=gen, device=DEV)[: rows // 20]
            emb[nz] = W._laplace(len(nz) * 768, 1e-4, gen, DEV).view(len(nz), 768)
        else:
            g[int(off[b]):int(off[b + 1])] = W._laplace(nb, 1e-4, gen, DEV)
    c = Case(g, off)
    c.step(ratio, bits)


@pytest.mark.parametrize("delta", [-5000, -1, 0, 1, 5000])
def test_threshold_at_the_boundary_between_zeros_and_values(path, delta):
    """A bucket of 2 M elements with k + delta non-zero ones (k = 200,000): the sample cannot tell
    whether the k-th largest magnitude is a zero, so a band from the smallest non-zero key up is
    staged and the exact counts decide.  Two steps, the second with the residual of the first."""
    n0, n1 = 2_000_000, 70_001
    ratio = 0.1
    k = int(np.floor(ratio * n0))
    gen = torch.Generator(device=DEV)
    gen.manual_seed(4242 + delta)
    g = torch.zeros(n0 + n1, device=DEV)
    pos = torch.randperm(n0, generator=gen, device=DEV)[: k + delta]
    v = W._laplace(k + delta, 1e-4, gen, DEV)
    v[v == 0] = 1e-4
    g[pos] = v
    g[n0:] = W._laplace(n1, 1e-4, gen, DEV)
    off = np.array([0, n0, n0 + n1], dtype=np.uint64)
    c = Case(g, off, chunk=256)
    c.step(ratio, 8)
    st = c.ctx.bucket_state(0)
    say("zero boundary", delta, path, st)
    if path == "auto":
        assert st["path"] == (3 if delta <= 0 else 2), st       # zero threshold / band, not the dense passes
    c.step(ratio, 4)


@pytest.mark.parametrize("span_tiles,seg_waves", [(1, 4), (2, 8), (4, 16), (8, 8), (16, 4), (16, 8), (16, 16), (2, 4)])
def test_streaming_geometries(monkeypatch, span_tiles, seg_waves):
    """The library picks tiles per workgroup and wavefronts per workgroup from the size of the
    gradient; the large-gradient shapes are forced here on a
    gradient the oracle sorts in a second: ragged buckets, last spans with fewer tiles than
    wavefronts, ties at the threshold, two error-feedback steps."""
    monkeypatch.setitem(nsml.Context.default_options, "span_tiles", int(span_tiles))
    monkeypatch.setitem(nsml.Context.default_options, "seg_waves", int(seg_waves))
    sizes = [200_003, 65_536 * 3 + 1, 4_099, 0, 333_333, 70_001]
    off = W.offsets_of(sizes)
    n = int(off[-1])
    say("geometry", span_tiles, seg_waves, n)
    g = _rand(n, 4242)
    g[5_000:9_000] = torch.round(g[5_000:9_000] * 2e3) / 2e3          # plateaus of equal magnitudes
    c = Case(g, off, chunk=512)
    c.step(0.02, 8)
    c.set_grad(_rand(n, 4243))
    c.step(0.004, 4)
    # ratios beyond an eighth: a band of keys is staged and the survivors come from the dense
    # accumulator; then a gradient that is mostly zeros, so that zeros must be sent (threshold key 0)
    c.set_grad(_rand(n, 4244))
    c.step(0.3, 8)
    g2 = _rand(n, 4245)
    g2[torch.rand(n, device=DEV, generator=torch.Generator(device=DEV).manual_seed(5)) < 0.7] = 0.0
    c.set_residual(np.zeros(n, dtype=np.float32))
    c.set_grad(g2)
    c.step(0.45, 32)


@pytest.mark.parametrize("span_tiles", [1, 2, 3, 4, 5, 7, 8, 12, 16])
def test_wavefront_per_tile_decompress_at_every_span_size(monkeypatch, span_tiles):
    """The decompress variant of the largest gradients (one wavefront per tile, 16 wavefronts per
    workgroup, which take 16 / span whole spans) forced on a small ragged gradient: last spans
    with fewer tiles than the others, a last workgroup with fewer spans, an empty bucket, sparse
    and crowded tiles, every value width."""
    monkeypatch.setitem(nsml.Context.default_options, "span_tiles", int(span_tiles))
    monkeypatch.setitem(nsml.Context.default_options, "decomp_variant", 1)
    sizes = [200_003, 65_536 * 3 + 1, 4_099, 0, 333_333, 70_001, 5]
    off = W.offsets_of(sizes)
    n = int(off[-1])
    say("wave-per-tile decompress, span", span_tiles, n)
    c = Case(_rand(n, 777), off, chunk=256)
    c.step(0.002, 4)
    c.set_grad(_rand(n, 778))
    c.step(0.05, 8)
    c.set_grad(_rand(n, 779))
    c.step(0.4, 16)
    c.set_grad(_rand(n, 780))
    c.step(1.0, 32)


@pytest.mark.parametrize("span_tiles", [0, 16])
@pytest.mark.parametrize("bits", [4, 8, 16, 32])
def test_decompress_of_a_malformed_index_list_stays_inside_the_output(monkeypatch, span_tiles, bits):
    """The kernels bound every index they are handed: a payload whose index list is not what
    compress writes (out of range, descending, repeated) gives unspecified values, but nothing
    outside the dense buffer is touched (sentinels on both sides stay intact), with both
    decompress variants and with decompress-accumulate."""
    if span_tiles:
        monkeypatch.setitem(nsml.Context.default_options, "span_tiles", int(span_tiles))
    sizes = [70_001, 3, 150_000, 0, 40_961]
    off = W.offsets_of(sizes)
    n = int(off[-1])
    ratio = 0.05
    ctx = nsml.Context(n, len(sizes), 256)
    idx, val, sc = ctx.alloc_payload(off, ratio, bits)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(99 + bits)
    pad = 8192
    for trial in range(3):
        raw = torch.randint(0, 2**31 - 1, (idx.numel(),), generator=gen, device=DEV, dtype=torch.int64)
        if trial == 1:
            raw = raw % 200_000                      # mostly inside some bucket, unordered, repeated
        if trial == 2:
            raw = torch.full_like(raw, -1)           # 0xFFFFFFFF everywhere
        idx.copy_(raw.to(idx.dtype))
        val.copy_(torch.randint(0, 256, (val.numel(),), generator=gen, device=DEV, dtype=torch.int64).to(val.dtype))
        if sc.numel():
            sc.copy_(torch.rand(sc.numel(), generator=gen, device=DEV))
        buf = torch.full((n + 2 * pad,), 7.0, device=DEV)
        dense = buf[pad:pad + n]
        ctx.decompress(idx, val, sc, n, off, ratio, bits, dense)
        ctx.decompress_accumulate(idx, val, sc, off, ratio, bits, dense)
        torch.cuda.synchronize()
        assert bool((buf[:pad] == 7.0).all()) and bool((buf[pad + n:] == 7.0).all())


def test_same_input_twice_gives_identical_bytes():
    """Determinism (the practical race detector): two runs, byte-identical outputs."""
    sizes = [300_000, 17, 200_003]
    off = W.offsets_of(sizes)
    n = int(off[-1])
    g = (_rand(n, 21) * 1e3).round() * 1e-3        # many ties
    outs = []
    for _ in range(2):
        ctx = nsml.Context(n, 3, 128)
        r = torch.zeros(n, device=DEV)
        idx, val, sc = ctx.compress(g, r, off, 0.03, 4)
        d = ctx.decompress(idx, val, sc, n, off, 0.03, 4)
        torch.cuda.synchronize()
        _, K, vb, ns = nsml.payload_layout(off, 0.03, 4, 128)
        outs.append([x.clone() for x in (idx[:K], val[:vb], sc[:ns], r, d)])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_context_reuse_across_layouts_and_ratios():
    """One context, changing bucket layout, ratio and width between calls."""
    ctx = nsml.Context(200_000, 8, 64)
    for i, (sizes, ratio, bits) in enumerate([([200_000], 0.01, 8), ([50_000] * 4, 0.2, 4),
                                              ([1, 199_999], 0.003, 16), ([200_000], 0.01, 8)]):
        off = W.offsets_of(sizes)
        c = Case(_rand(200_000, 40 + i), off, chunk=64, ctx=ctx)
        c.step(ratio, bits)


def test_two_contexts_on_two_streams_at_once(path):
    """Two contexts working at the same time on streams of their own (the header allows it): with
    every bucket on the dense passes both run the launch whose workgroups meet at barriers, so
    the two teams must fit the device together.  Results of both against the oracle, five rounds."""
    n = 3_000_000
    off = W.offsets_of([1_000_000, 1_500_001, 499_999])
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    cases = []
    for i in range(2):
        g = _rand(n, 4000 + i)
        cases.append({"ctx": nsml.Context(n, 3, 256), "g": g, "r": torch.zeros(n, device=DEV),
                      "g_h": g.cpu().numpy(), "r_h": np.zeros(n, dtype=np.float32)})
    torch.cuda.synchronize()
    for rnd in range(5):
        ratio, bits = [(0.01, 8), (0.3, 4), (0.05, 16), (1.0, 8), (0.002, 4)][rnd]
        outs = []
        for i, c in enumerate(cases):
            with torch.cuda.stream(streams[i]):
                outs.append(c["ctx"].compress(c["g"], c["r"], off, ratio, bits))
        torch.cuda.synchronize()
        for c, (idx, val, sc) in zip(cases, outs):
            c["ctx"].path_stats()
            want = oracle.compress(c["g_h"], c["r_h"], off, ratio, bits, 256, nthreads=8)
            k_b, K, vb, ns = oracle.layout(off, ratio, bits, 256)
            got = (idx.cpu().numpy().view(np.uint32)[:K], val.cpu().numpy()[:vb], sc.cpu().numpy()[:ns])
            from gpu_util import compare_payload
            compare_payload(off, ratio, bits, 256, got, want)
            assert np.array_equal(c["r"].cpu().numpy().view(np.uint32), c["r_h"].view(np.uint32))
    for c in cases:
        c["ctx"].close()


def test_gpu_argument_errors():
    ctx = nsml.Context(10_000, 2, 64)
    g = _rand(10_000, 1)
    r = torch.zeros_like(g)
    off = W.offsets_of([10_000])
    with pytest.raises(nsml.NsmlError) as e:
        ctx.compress(g, r, off, 0.0, 8)
    assert e.value.code == nsml.EINVAL
    with pytest.raises(nsml.NsmlError) as e:
        ctx.compress(g, r, W.offsets_of([3_000, 3_000, 4_000]), 0.5, 8)    # 3 buckets > max 2
    assert e.value.code == nsml.ECAP
    big = _rand(20_000, 2)
    with pytest.raises(nsml.NsmlError) as e:
        ctx.compress(big, torch.zeros_like(big), W.offsets_of([20_000]), 0.5, 8)
    assert e.value.code == nsml.ECAP
    with pytest.raises(nsml.NsmlError) as e:
        ctx.compress(g[1:], r[1:], W.offsets_of([9_999]), 0.5, 8)          # misaligned
    assert e.value.code == nsml.EINVAL
    with pytest.raises(ValueError):                                        # the binding's own size check
        ctx.compress(g, r[:-1], off, 0.5, 8)


def test_l2norm_byproduct():
    """The streaming pass also returns |grad|_2 (density test of Algorithm 2 Step 1): within
    1e-6 relative of the oracle's double-precision norm, per bucket and in total, and the same
    bits on a second run."""
    sizes = [1, 64, 4097, 0, 300_003, 7, 1_000_001]
    off = W.offsets_of(sizes)
    n = int(off[-1])
    g = _rand(n, 77, sigma=3e-3)
    ctx = nsml.Context(n, len(sizes), 64)
    got = []
    for _ in range(2):
        r = _rand(n, 78)
        ctx.compress(g, r, off, 0.01, 8)
        got.append(ctx.last_l2norm(len(sizes)))
    want_tot, want_per = oracle.l2norm(g.cpu().numpy(), off)
    tot, per = got[0]
    assert abs(tot - want_tot) <= 1e-6 * want_tot
    assert np.all(np.abs(per - want_per) <= 1e-6 * np.maximum(want_per, 1e-30))
    assert per[3] == 0.0
    assert got[0][0] == got[1][0] and np.array_equal(got[0][1], got[1][1])


@pytest.mark.parametrize("bits", [4, 8, 16, 32])
def test_decompress_accumulate(bits):
    """Three workers' payloads summed into one dense buffer, bit-exact against the oracle."""
    sizes = [5, 70_000, 0, 33_333, 100_001]
    off = W.offsets_of(sizes)
    n = int(off[-1])
    ctx = nsml.Context(n, len(sizes), 64)
    dense = torch.full((n,), 0.125, device=DEV)
    want = np.full(n, 0.125, dtype=np.float32)
    for w in range(3):
        g = _rand(n, 300 + w, sigma=1e-2)
        r = torch.zeros(n, device=DEV)
        idx, val, sc = ctx.compress(g, r, off, 0.03, bits)
        ctx.decompress_accumulate(idx, val, sc, off, 0.03, bits, dense)
        w_idx, w_val, w_sc = oracle.compress(g.cpu().numpy(), np.zeros(n, np.float32), off, 0.03, bits, 64)
        oracle.decompress_accumulate(w_idx, w_val, w_sc, want, off, 0.03, bits, 64)
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), want.view(np.uint32))


def test_hip_graph_capture_and_replay(path):
    """A compress + decompress step captured in a HIP graph (no memset nodes, no host
    synchronisation once the tables exist) replays correctly: three replays with fresh gradients
    copied into the captured buffers, program-owned eager work in between, each replay compared
    with an eager run on a second context."""
    sizes = [70_000, 3, 131_072, 40_001]
    off = W.offsets_of(sizes)
    n = int(off[-1])
    ratio, bits = 0.02, 4
    ctx_g, ctx_e = nsml.Context(n, len(sizes), 256), nsml.Context(n, len(sizes), 256)
    g_static = _rand(n, 500)
    r_static = torch.zeros(n, device=DEV)
    idx, val, sc = ctx_g.alloc_payload(off, ratio, bits)
    dense = torch.zeros(n, device=DEV)
    # one eager call builds the tables (that part synchronises and cannot be captured)
    ctx_g.compress(g_static, r_static, off, ratio, bits, idx, val, sc)
    ctx_g.decompress(idx, val, sc, n, off, ratio, bits, dense)
    torch.cuda.synchronize()
    r_static.zero_()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            ctx_g.compress(g_static, r_static, off, ratio, bits, idx, val, sc)
            ctx_g.decompress(idx, val, sc, n, off, ratio, bits, dense)
    torch.cuda.synchronize()
    r_static.zero_()
    r_eager = torch.zeros(n, device=DEV)
    _, K, vb, ns = nsml.payload_layout(off, ratio, bits, 256)
    for rep in range(3):
        g_new = _rand(n, 600 + rep)
        g_static.copy_(g_new)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        e_idx, e_val, e_sc = ctx_e.compress(g_new, r_eager, off, ratio, bits)
        e_dense = ctx_e.decompress(e_idx, e_val, e_sc, n, off, ratio, bits)
        torch.cuda.synchronize()
        assert torch.equal(idx[:K], e_idx[:K]) and torch.equal(val[:vb], e_val[:vb])
        assert torch.equal(sc[:ns], e_sc[:ns])
        assert torch.equal(r_static, r_eager) and torch.equal(dense, e_dense)
        (g_new * 2).sum().item()          # unrelated eager work and a synchronisation between replays


def test_internal_error_is_reported_by_the_next_call_once():
    """A tripped device-side consistency check is reported by the next GPU entry point called on
    the context (which enqueues nothing) and then cleared; raised here through the diagnostic
    option, since no input makes the check fail."""
    g, off = W.cfg1(DEV)
    c = Case(g, off)
    c.step(0.01, 8)
    c.ctx.set_option("trip_check", 1)
    r_before = c.r.clone()
    with pytest.raises(nsml.NsmlError) as e:
        c.ctx.compress(c.g, c.r, off, 0.01, 8)
    assert e.value.code == nsml.EINTERNAL
    torch.cuda.synchronize()
    assert torch.equal(c.r, r_before)                 # nothing ran
    c.step(0.01, 8)                                   # reported once: the context works again
    c.ctx.set_option("trip_check", 1)
    with pytest.raises(nsml.NsmlError) as e:
        c.ctx.path_stats()
    assert e.value.code == nsml.EINTERNAL
    with pytest.raises(nsml.NsmlError):
        c.ctx.decompress(*c.ctx.alloc_payload(off, 0.01, 8), c.n, off, 0.01, 8)
    with pytest.raises(nsml.NsmlError):
        c.ctx.set_option("no_such_option", 1)
    with pytest.raises(nsml.NsmlError):
        c.ctx.set_option("span_tiles", 17)


def test_context_sized_for_a_maximum_ratio():
    """nsml_create_ex: the survivor-value buffer is sized by max_ratio; larger ratios are refused."""
    sizes = [300_000, 5, 70_001]
    off = W.offsets_of(sizes)
    n = int(off[-1])
    full = nsml.Context(n, len(sizes), 2048)
    small = nsml.Context(n, len(sizes), 2048, max_ratio=0.1)
    assert full.workspace_bytes - small.workspace_bytes >= int(0.85 * 4 * n)
    c = Case(_rand(n, 77), off, ctx=small)
    c.step(0.1, 8)
    c.step(0.03, 4)
    with pytest.raises(nsml.NsmlError) as e:
        small.compress(c.g, c.r, off, 0.11, 8)
    assert e.value.code == nsml.ECAP
