"""slim_dequant_matmul_noalloc (the entry point for callers that cannot allocate device memory) against
slim_dequant_matmul, through the C ABI: two calls in a row, the second on a smaller layer, must give bit for bit
the existing entry point's output (same kernels, same launch shapes; the partial sums live in the library's fixed
buffer instead of the context's workspace), and both agree with the float64 oracle within the bound of the linear
layer's parity test.  A layer whose partial sums exceed the fixed buffer is rejected with a clear error."""
import numpy as np
import pytest
import torch

from oracle import slim_oracle as orc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def slim():
    from paper_2405_14917_amd import binding
    s = binding.Slim("cuda:0")
    yield s
    s.close()


def stored_layer(slim, seed, n, m, beta, N):
    """A stored layer built from seeded random codes through slim_pack: widths N-1, N, N+1 in equal numbers."""
    rng = np.random.default_rng(seed)
    k = m // beta
    bits = np.full(k, N, dtype=np.uint8)
    bits[0::4] = N - 1
    bits[1::4][: bits[0::4].size] = N + 1
    codes = np.zeros((n, m), dtype=np.uint8)
    for g in range(k):
        codes[:, g * beta:(g + 1) * beta] = rng.integers(0, 2 ** int(bits[g]), (n, beta), dtype=np.uint8)
    scale = rng.uniform(0.005, 0.02, (n, k))
    zero = np.rint(rng.uniform(0, 2.0 ** bits.astype(np.float64)[None, :] - 1, (n, k)))
    packed, gbits, row_off, _ = slim.pack(torch.from_numpy(codes).cuda(), torch.from_numpy(bits).cuda(), beta)
    return dict(packed=packed, gbits=gbits, row_off=row_off, scale=torch.from_numpy(scale).cuda(),
                zero=torch.from_numpy(zero).cuda(), beta=beta, n=n, m=m)


def both_ways(slim, L, t_x, seed):
    rng = np.random.default_rng(seed)
    X = torch.from_numpy(rng.standard_normal((t_x, L["m"])).astype(np.float16)).cuda()
    args = (L["packed"], L["gbits"], L["row_off"], L["scale"], L["zero"], L["beta"], X)
    Y_ref = slim.dequant_matmul(*args)
    Y = torch.full((t_x, L["n"]), float("nan"), dtype=torch.float32, device="cuda")
    slim.dequant_matmul(*args, Y=Y, noalloc=True)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y_ref), "the two entry points differ"
    h = lambda t: t.cpu().numpy()
    Yo = orc.dequant_matmul(h(L["packed"]).view(np.uint32), h(L["gbits"]).view(np.uint32), h(L["row_off"]),
                            h(L["scale"]), h(L["zero"]), L["beta"], h(X).astype(np.float64))
    codes, _ = orc.unpack(h(L["packed"]).view(np.uint32), h(L["gbits"]).view(np.uint32), L["beta"], L["m"] // L["beta"])
    What = np.repeat(h(L["scale"]), L["beta"], axis=1) * (codes - np.repeat(h(L["zero"]), L["beta"], axis=1))
    bound = np.abs(h(X).astype(np.float64)) @ np.abs(What).T
    assert np.all(np.abs(h(Y) - Yo) <= 1e-5 * bound + 1e-30), "differs from the oracle"


def test_noalloc_equals_the_existing_entry_point_twice_in_a_row(slim):
    ws0 = slim.workspace_bytes()
    big = stored_layer(slim, 1, 1024, 2048, 128, 2)       # several group ranges: the fixed buffer is in use
    small = stored_layer(slim, 2, 384, 512, 64, 3)        # a smaller layer right after it: stale contents must not show
    both_ways(slim, big, 8, 3)
    both_ways(slim, small, 3, 4)
    both_ways(slim, big, 1, 5)
    # the calls of the new entry point leave the context's workspace alone (the existing one may have grown it)
    ws1 = slim.workspace_bytes()
    Y = torch.empty((8, big["n"]), dtype=torch.float32, device="cuda")
    X = torch.zeros((8, big["m"]), dtype=torch.float16, device="cuda")
    slim.dequant_matmul(big["packed"], big["gbits"], big["row_off"], big["scale"], big["zero"], big["beta"], X, Y=Y,
                        noalloc=True)
    assert slim.workspace_bytes() == ws1 >= ws0


def test_noalloc_rejects_a_layer_beyond_its_buffer(slim):
    from paper_2405_14917_amd import binding
    n, m, beta, t_x = 98304, 4096, 128, 16               # 3 group ranges x 16 tokens x 98304 rows > 4 Mi floats
    k = m // beta
    packed = torch.zeros((m * 2 // 32, n), dtype=torch.int32, device="cuda")
    gbits = torch.full(((k + 15) // 16,), 0x55555555, dtype=torch.int32, device="cuda")       # every group 2 bits wide
    row_off = (torch.arange(k + 1, dtype=torch.int32) * (beta * 2 // 32)).cuda()
    scale = torch.ones((n, k), dtype=torch.float64, device="cuda")
    zero = torch.zeros((n, k), dtype=torch.float64, device="cuda")
    X = torch.ones((t_x, m), dtype=torch.float16, device="cuda")
    Y = torch.full((t_x, n), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(binding.SlimError) as e:
        slim.dequant_matmul(packed, gbits, row_off, scale, zero, beta, X, Y=Y, noalloc=True)
    assert e.value.status == binding.ERR_UNSUPPORTED and "fixed buffer" in str(e.value)
    torch.cuda.synchronize()
    assert bool((Y == 7.0).all()), "a rejected call must not touch its output"
    # the same layer goes through the allocating entry point
    slim.dequant_matmul(packed, gbits, row_off, scale, zero, beta, X, Y=Y)
    torch.cuda.synchronize()
    assert bool((Y == 0.0).all())
