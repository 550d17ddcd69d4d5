"""Parity at the FULL sizes of the benchmark configurations, in the launch configuration bench.py times: same
generators, same call sequence, same sizes.

  C2  LLaMA-7B q_proj shape     4096 x  4096, 131072 tokens
  C3  LLaMA-7B down_proj shape  4096 x 11008, 262144 tokens   (the headline workload of bench.py)
  C4  LLaMA-13B up_proj shape  13824 x  5120, 262144 tokens, widths {2, 3, 4}
  C5  LLaMA-70B-shaped layer   28672 x  8192, 262144 tokens

The oracle cannot run a whole pass of these sizes in seconds, so each stage is checked on outputs the oracle can
compute one by one (sampled Gram rows, the whole inverse, sampled SBA candidates, sampled rows of the sweep in the
row-independent mask scope, the packed words bit for bit) or through identities that hold at any size.  Stage inputs
that are results of an earlier stage are computed by the ORACLE (from the first chunk of tokens where the full set
would take minutes), never taken from the HIP path.  On C2 the default block-wide mask scope is also compared code
for code over the whole layer."""
import concurrent.futures
import os
import time

import numpy as np
import pytest
import torch

from oracle import slim_oracle as orc
from paper_2405_14917_amd import synth

pytestmark = pytest.mark.gpu

MARGIN = 1e-6
T_SBA = 2048
NAMES = ["C2", "C3", "C4", "C5"]


@pytest.fixture(scope="module")
def slim():
    from paper_2405_14917_amd import binding
    s = binding.Slim("cuda:0")
    yield s
    s.close()


def say(msg):
    print("[full-size %s] %s" % (time.strftime("%H:%M:%S"), msg), flush=True)


@pytest.fixture(scope="module", params=NAMES)
def layer(request):
    """W, X on the host (fp16) and on the device, plus the oracle's second-order information from the first chunk
    of tokens (the oracle's Gram matrix over all tokens would take minutes)."""
    cfg = synth.CONFIGS[request.param]
    say("%s: generating W %dx%d and X %dx%d" % (cfg.name, cfg.n, cfg.m, cfg.m, cfg.t))
    W = synth.make_weights(cfg)
    Xd = torch.empty((cfg.m, cfg.t), dtype=torch.float16, device="cuda")
    chunks = []
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 8)) as pool:
        for c, xc in enumerate(pool.map(lambda i: synth.activation_chunk(cfg, i), range(synth.n_chunks(cfg)))):
            chunks.append(xc)
            Xd[:, c * synth.CHUNK_TOKENS:c * synth.CHUNK_TOKENS + xc.shape[1]] = torch.from_numpy(xc).cuda()
    say("%s: oracle Gram matrix of the first chunk and its inverse (m = %d)" % (cfg.name, cfg.m))
    G0 = np.zeros((cfg.m, cfg.m))
    orc.gram_accumulate(G0, chunks[0])
    G32 = G0.astype(np.float32)
    G32 = np.maximum(G32, G32.T)
    del G0
    t0 = chunks[0].shape[1]
    U, d, lam = orc.hessian_inverse(G32.astype(np.float64), t0, cfg.percdamp)
    _, grp, _ = orc.salience(W, d, cfg.beta)
    say("%s: inputs ready" % cfg.name)
    L = dict(cfg=cfg, W=W, chunks=chunks, Wd=torch.from_numpy(W).cuda(), Xd=Xd, G32=G32, t0=t0, U=U, d=d, lam=lam,
             grp=grp)
    del W, chunks, Xd, G32, U, d, grp
    yield L
    L.clear()
    torch.cuda.empty_cache()


def host(t):
    return t.detach().cpu().numpy()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_gram_sampled_rows(slim, layer):
    cfg = layer["cfg"]
    G = torch.zeros((cfg.m, cfg.m), dtype=torch.float32, device="cuda")
    nt = slim.hessian_accumulate(layer["Xd"], G, 0)          # one call over all tokens, as bench.py does
    assert nt == cfg.t
    Gg = host(G).astype(np.float64)
    assert np.array_equal(Gg, Gg.T)
    rng = np.random.default_rng(0)
    # rows from every part of the matrix: random ones, outlier channels, the first and last tile rows
    rows = np.unique(np.concatenate([rng.integers(0, cfg.m, 10), synth.outlier_activation_channels(cfg)[:4],
                                     [0, 255, 256, cfg.m - 257, cfg.m - 1]]))
    ref = np.zeros((rows.size, cfg.m))
    diag = np.zeros(cfg.m)
    for xc in layer["chunks"]:
        x = xc.astype(np.float64)
        ref += x[rows] @ x.T
        diag += np.einsum("ij,ij->i", x, x)
    assert np.allclose(np.diag(Gg), diag, rtol=2e-5)
    scale = np.sqrt(np.outer(diag[rows], diag))
    err = np.max(np.abs(Gg[rows] - ref) / scale)
    say("%s gram: max scaled error on %d sampled rows %.3e" % (cfg.name, rows.size, err))
    assert err < 2e-6 * np.sqrt(cfg.t / 512)


def test_inverse_full_size(slim, layer):
    cfg = layer["cfg"]
    U, d = slim.hessian_inverse(dev(layer["G32"]), layer["t0"], cfg.percdamp)
    U, d = host(U), host(d)
    assert np.all(np.tril(U, -1) == 0.0)
    err = np.linalg.norm(U - layer["U"]) / np.linalg.norm(layer["U"])
    say("%s inverse: relative Frobenius distance of U from the oracle's %.3e" % (cfg.name, err))
    assert err < 1e-9
    assert np.allclose(d, layer["d"], rtol=1e-8)


def test_salience_full_size(slim, layer):
    cfg = layer["cfg"]
    col, grp, _ = slim.salience(layer["Wd"], dev(layer["d"]), cfg.beta)
    assert np.allclose(host(grp), layer["grp"], rtol=1e-11)


def test_sba_sampled_candidates(slim, layer):
    cfg = layer["cfg"]
    k = cfg.k
    Xs_d = layer["Xd"][:, :T_SBA]
    bits, p_star, obj = slim.sba_allocate(layer["Wd"], dev(layer["grp"]), cfg.beta, cfg.N, Xs_d)
    assert obj.shape == (k // 2 + 1,)
    W = layer["W"].astype(np.float64)
    Xs = layer["chunks"][0][:, :T_SBA].astype(np.float64)
    order = np.argsort(layer["grp"], kind="stable")
    Y = Xs.T @ W.T
    for p in sorted({0, k // 4, p_star, k // 2}):
        Wp = orc.rtn_fakequant_fast(W, orc.bits_for_p(order, k, cfg.N, p), cfg.beta)
        ref = orc.softmax_kl(Y, Xs.T @ Wp.T)
        say("%s SBA candidate %d: objective %.12e, oracle %.12e" % (cfg.name, p, obj[p], ref))
        assert obj[p] == pytest.approx(ref, rel=1e-9), "objective of candidate %d" % p
    assert p_star == int(np.argmin(obj))
    gap = np.sort(obj)[1] - np.sort(obj)[0]
    if gap > MARGIN * obj.min():
        assert np.array_equal(host(bits), orc.bits_for_p(order, k, cfg.N, p_star))
    else:
        say("%s SBA: the two best candidates lie within the margin, the widths are not compared" % cfg.name)
    b = host(bits).astype(int)
    assert b.sum() == cfg.N * k and (b == cfg.N - 1).sum() == (b == cfg.N + 1).sum() == p_star


def _alloc_bits(cfg):
    """A fixed allocation with all three widths: every seventh group narrower, as many groups wider."""
    k = cfg.k
    bits = np.full(k, cfg.N, dtype=np.uint8)
    lo = np.arange(3, k, 7)
    hi = np.arange(0, k, 7)[:lo.size]
    bits[lo] = cfg.N - 1
    bits[hi] = cfg.N + 1
    assert int(bits.astype(int).sum()) == cfg.N * k
    return bits


def test_sweep_sampled_rows_identities_and_packing(slim, layer):
    from paper_2405_14917_amd import binding
    cfg = layer["cfg"]
    beta, k = cfg.beta, cfg.k
    bits = _alloc_bits(cfg)
    Ud, W = dev(layer["U"]), layer["W"]
    # (1) row-independent mask scope: the oracle reproduces sampled rows one by one
    rows = np.sort(np.random.default_rng(1).choice(cfg.n, 48, replace=False))
    out = slim.gptq_quantize(layer["Wd"], Ud, dev(bits), beta, params=binding.make_params(mask_scope=orc.SCOPE_ROW),
                             want_what=torch.float64)
    ref = orc.gptq_quantize(W[rows], layer["U"], bits, beta, orc.tau_grid(), scope=orc.SCOPE_ROW)
    ok = (ref["round_margin"].min(axis=1) > MARGIN) & (ref["sqc_margin"].min(axis=1) > MARGIN)
    say("%s sweep: %d of %d sampled rows have every decision outside the margin" % (cfg.name, ok.sum(), ok.size))
    assert ok.mean() > 0.75
    codes = host(out["codes"][rows])
    assert np.array_equal(codes[ok], ref["codes"][ok])
    What = host(out["What"][rows])
    assert np.linalg.norm(What[ok] - ref["What"][ok]) / np.linalg.norm(ref["What"][ok]) < 1e-10
    assert np.allclose(host(out["scale"][rows])[ok], ref["scale"][ok], rtol=1e-12)
    assert np.array_equal(host(out["zero"][rows])[ok], ref["zero"][ok])
    del out
    # (2) default block-wide scope: identities that hold at any size
    out = slim.gptq_quantize(layer["Wd"], Ud, dev(bits), beta, want_what=torch.float64, want_sum_e2=True)
    codes, What = host(out["codes"]), host(out["What"])
    scale, zero = host(out["scale"]), host(out["zero"])
    assert all(codes[:, g * beta:(g + 1) * beta].max() < 2 ** int(bits[g]) for g in range(k))
    for g in range(0, k, max(1, k // 8)):          # W_hat is the dequantised code, group by group
        deq = scale[:, g:g + 1] * (codes[:, g * beta:(g + 1) * beta] - zero[:, g:g + 1])
        assert np.allclose(What[:, g * beta:(g + 1) * beta], deq, rtol=1e-15, atol=0)
    G = layer["G32"].astype(np.float64)
    dW = W.astype(np.float64) - What
    dWG = dW @ G
    # sum of the squared compensation errors = tr(dW (H + lambda I) dW^T)  (W - W_hat = E U, U (H + lambda I) U^T = I)
    tr = 2.0 / layer["t0"] * float(np.sum(dWG * dW)) + layer["lam"] * float(np.sum(dW * dW))
    assert host(out["sum_e2"])[0] == pytest.approx(tr, rel=1e-7)
    # the compensated result beats round-to-nearest on the same grids in the layer-output error
    rtn = np.empty_like(What)
    for g in range(k):
        s, z = scale[:, g:g + 1], zero[:, g:g + 1]
        blk = W[:, g * beta:(g + 1) * beta].astype(np.float64)
        q = (blk >= 0).astype(np.float64) if bits[g] == 1 else np.clip(np.rint(blk / s) + z, 0, 2 ** int(bits[g]) - 1)
        rtn[:, g * beta:(g + 1) * beta] = s * (q - z)
    dR = W.astype(np.float64) - rtn
    assert float(np.sum(dWG * dW)) < float(np.sum((dR @ G) * dR))
    del dWG, dW, dR, rtn, What
    # (3) packing of these codes, bit for bit
    base = orc.bit_base_for(cfg.N)
    packed, gbits, row_off, m_star = slim.pack(out["codes"], dev(bits), beta, bit_base=base)
    po, go, ro, mo = orc.pack_fast(codes, bits, beta, base)
    assert m_star == mo == cfg.m * cfg.N // 32
    assert np.array_equal(host(row_off), ro) and np.array_equal(host(gbits).view(np.uint32), go)
    assert np.array_equal(host(packed).view(np.uint32), po)


def test_default_scope_sweep_code_for_code(slim, layer):
    """The default block-wide mask scope over the WHOLE layer against the oracle, fed with the oracle's U and a
    fixed allocation: every code, scale and zero of every row whose decisions lie outside the margin."""
    cfg = layer["cfg"]
    if cfg.name != "C2":
        pytest.skip("the oracle's full sweep takes minutes beyond C2; the larger shapes are covered row by row")
    bits = _alloc_bits(cfg)
    out = slim.gptq_quantize(layer["Wd"], dev(layer["U"]), dev(bits), cfg.beta, want_what=torch.float64)
    t0 = time.perf_counter()
    ref = orc.gptq_quantize(layer["W"], layer["U"], bits, cfg.beta, orc.tau_grid())
    say("C2 default-scope sweep: the oracle took %.1f s" % (time.perf_counter() - t0))
    ok = (ref["round_margin"].min(axis=1) > MARGIN) & (ref["sqc_margin"].min(axis=1) > MARGIN)
    codes = host(out["codes"])
    equal = float((codes == ref["codes"]).mean())
    fro = np.linalg.norm(host(out["What"]) - ref["What"]) / np.linalg.norm(ref["What"])
    say("C2 default-scope sweep: %d of %d rows outside the margin, equal codes %.6f, ||What - What_o||_F / ||What_o||_F "
        "= %.3e" % (ok.sum(), ok.size, equal, fro))
    assert ok.mean() > 0.75
    assert np.array_equal(codes[ok], ref["codes"][ok])
    assert np.allclose(host(out["scale"])[ok], ref["scale"][ok], rtol=1e-12)
    assert np.array_equal(host(out["zero"])[ok], ref["zero"][ok])
    assert fro < 1e-3


def test_chained_pass_from_the_same_gram_matrix(slim, layer):
    """The whole C2 layer end to end behind the Gram matrix: the HIP path's inverse, salience, bit allocation and sweep,
    each on the HIP path's own earlier results, against the oracle's steps in the same order, both started from the
    SAME Gram matrix (the HIP path's, over all 131072 tokens).  Behind the Gram matrix both sides work in fp64, so the
    the benchmark spec's end-to-end bar is asserted as it stands: dequantised weights within 1e-3 in relative Frobenius norm
    (the pass from X on differs from the oracle's by the fp32 accumulation of the Gram matrix alone)."""
    cfg = layer["cfg"]
    if cfg.name != "C2":
        pytest.skip("a whole oracle pass takes minutes beyond C2; the reduced shapes run the same chain")
    Wd, Xd, W = layer["Wd"], layer["Xd"], layer["W"]
    G = torch.zeros((cfg.m, cfg.m), dtype=torch.float32, device="cuda")
    nt = slim.hessian_accumulate(Xd, G, 0)
    U, d = slim.hessian_inverse(G, nt, cfg.percdamp)
    _, grp, _ = slim.salience(Wd, d, cfg.beta)
    bits, p_star, obj = slim.sba_allocate(Wd, grp, cfg.beta, cfg.N, Xd[:, :T_SBA])
    out = slim.gptq_quantize(Wd, U, bits, cfg.beta, want_what=torch.float64)
    t0 = time.perf_counter()
    W64 = W.astype(np.float64)
    Uo, do, _ = orc.hessian_inverse(host(G).astype(np.float64), nt, cfg.percdamp)
    _, grp_o, _ = orc.salience(W64, do, cfg.beta)
    assert layer["chunks"][0].shape[1] >= T_SBA
    Xs = layer["chunks"][0][:, :T_SBA].astype(np.float64)
    bits_o, p_o, obj_o, margin_o = orc.sba_allocate(W64, grp_o, cfg.beta, cfg.N, Xs)
    ref = orc.gptq_quantize(W64, Uo, bits_o, cfg.beta, orc.tau_grid(), hinv_diag=do)
    say("C2 chained pass: the oracle's steps took %.1f s" % (time.perf_counter() - t0))
    assert np.linalg.norm(host(U) - Uo) / np.linalg.norm(Uo) < 1e-9
    assert np.allclose(host(grp), grp_o, rtol=1e-9)
    assert np.allclose(obj, obj_o, rtol=1e-8)
    if margin_o > MARGIN:
        assert p_star == p_o
    assert np.array_equal(host(bits), bits_o)
    codes = host(out["codes"])
    ok = (ref["round_margin"].min(axis=1) > MARGIN) & (ref["sqc_margin"].min(axis=1) > MARGIN)
    equal = float((codes == ref["codes"]).mean())
    fro = np.linalg.norm(host(out["What"]) - ref["What"]) / np.linalg.norm(ref["What"])
    say("C2 chained pass from the same Gram matrix: p* = %d, %d of %d rows outside the margin, equal codes %.6f, "
        "||What - What_o||_F / ||What_o||_F = %.3e" % (p_star, ok.sum(), ok.size, equal, fro))
    assert np.array_equal(codes[ok], ref["codes"][ok])
    assert fro <= 1e-3


def test_learnable_clipping_full_size(slim, layer):
    """SliM-LLM+ (learnable weight clipping, three AdamW steps) on the whole layer against the oracle, fed with the
    oracle-side Gram matrix and a fixed allocation."""
    cfg = layer["cfg"]
    if cfg.name != "C2":
        pytest.skip("three oracle steps on the larger shapes take minutes; C2 exercises the same kernels at full width")
    bits = _alloc_bits(cfg)
    steps = 3
    t0 = time.perf_counter()
    ref = orc.lwc_quantize(layer["W"], layer["G32"].astype(np.float64), layer["t0"], bits, cfg.beta, steps=steps)
    say("C2 learnable clipping: the oracle took %.1f s" % (time.perf_counter() - t0))
    out = slim.lwc_quantize(layer["Wd"], dev(layer["G32"]), layer["t0"], dev(bits), cfg.beta, steps=steps,
                            want_what=torch.float64)
    assert np.allclose(out["loss_curve"], ref["loss_curve"], rtol=1e-9)
    ok = ref["round_margin"].min(axis=1) > MARGIN
    say("C2 learnable clipping: %d of %d rows outside the margin, loss %s" % (ok.sum(), ok.size, out["loss_curve"]))
    assert ok.mean() > 0.75
    assert np.array_equal(host(out["codes"])[ok], ref["codes"][ok])
    assert np.allclose(host(out["scale"]), ref["scale"], rtol=1e-9)
    assert np.linalg.norm(host(out["What"])[ok] - ref["What"][ok]) / np.linalg.norm(ref["What"][ok]) < 1e-8


def test_pass_as_timed_equals_the_entry_points_one_by_one(slim, layer):
    """The driver bench.py times (two contexts on two streams, the first half of the bit allocation beside the
    inverse in the persistent part-of-the-chip form, no host outputs, the inverse returning with its triangular
    inverse in flight) gives bit for bit what the entry points give when called one after the other on one context."""
    from paper_2405_14917_amd import binding, pipeline
    cfg = layer["cfg"]
    Wd, Xd = layer["Wd"], layer["Xd"]
    base = binding.bit_base_for(cfg.N)
    drv = pipeline.LayerPass(slim, cfg.m, cfg.beta, cfg.N, cfg.percdamp, t_sba=T_SBA)
    try:
        r1 = drv.run(Wd, Xd)
        r2 = drv.run(Wd, Xd)                                   # and it is reproducible
        G = torch.zeros((cfg.m, cfg.m), dtype=torch.float32, device="cuda")
        nt = slim.hessian_accumulate(Xd, G, 0)
        U, d = slim.hessian_inverse(G, nt, cfg.percdamp)
        _, grp, _ = slim.salience(Wd, d, cfg.beta)
        bits, p_star, _ = slim.sba_allocate(Wd, grp, cfg.beta, cfg.N, Xd[:, :T_SBA])
        out = slim.gptq_quantize(Wd, U, bits, cfg.beta)
        packed, gbits, row_off, m_star = slim.pack(out["codes"], bits, cfg.beta, bit_base=base)
        assert torch.equal(U, drv.U) and torch.equal(d, drv.d)
        for r in (r1, r2):
            assert int(r["p_star"]) == p_star and int(r["m_star"]) == m_star
            assert torch.equal(r["bits"], bits) and torch.equal(r["codes"], out["codes"])
            assert torch.equal(r["scale"], out["scale"]) and torch.equal(r["zero"], out["zero"])
            assert torch.equal(r["packed"][:m_star], packed) and torch.equal(r["row_off"], row_off)
        say("%s whole pass: p* = %d, m* = %d" % (cfg.name, p_star, m_star))
    finally:
        drv.close()
