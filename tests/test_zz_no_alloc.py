"""GPU test of the entry point that allocates nothing (hbl_bitlinear_forward_small): through the C ABI, against
the workspace-carrying forward calls on the same inputs - bit for bit - on calls in a row that share the
library's static device scratch, the later ones smaller than the first."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2504_18415_amd import synth

pytestmark = pytest.mark.gpu

EPS = 1e-5


@pytest.fixture(scope="module")
def hbl():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2504_18415_amd import hbl as H
    H.lib()
    return H


def dev_x(x_np):
    if x_np.dtype == np.uint16:
        return torch.from_numpy(x_np.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(x_np).cuda()


def problem(hbl, name, T, K, N, hadamard, groups, seed, dtype=synth.BF16):
    site = synth.Site(name, T, K, N, hadamard=hadamard, groups=groups, x_dtype=dtype, outlier_frac=0.01,
                      outlier_scale=30.0, seed=seed)
    x = dev_x(synth.make_x(site))
    W = torch.from_numpy(synth.make_w(site)).cuda()
    rows = N // groups
    codes, alphas = zip(*[hbl.ternarize_weights_absmean(W[g * rows:(g + 1) * rows].contiguous(), EPS)
                          for g in range(groups)])
    packed = hbl.pack_ternary_2bit(torch.cat(codes, 0).contiguous())
    return site, x, packed, torch.cat(alphas).contiguous()


def test_no_alloc_forward_matches_workspace_forward(hbl):
    # a large problem first (split K range: partial tiles in the scratch), then smaller ones that reuse its
    # scratch while the old contents are still there, then the large one again
    cases = [("a", 64, 16384, 1056, True, 1, 4, 101), ("b", 5, 4096, 288, False, 3, 4, 102),
             ("c", 33, 2048, 96, True, 1, 8, 103), ("d", 1, 512, 32, True, 1, 4, 104),
             ("a2", 64, 16384, 1056, True, 1, 4, 101), ("e", 16, 4096, 12288, False, 3, 4, 105)]
    for name, T, K, N, hadamard, groups, bits, seed in cases:
        print(f"[gpu-case] no-alloc forward {name}: T={T} K={K} N={N} hadamard={hadamard} bits={bits}", flush=True)
        site, x, packed, alphas = problem(hbl, name, T, K, N, hadamard, groups, seed)
        fn = hbl.hbitlinear_forward if hadamard else hbl.plain_bitlinear_forward
        want = fn(x, packed, N, alphas, bits, EPS)
        y = torch.full((T, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        before = torch.cuda.memory_allocated()
        hbl.bitlinear_forward_small(x, packed, N, alphas, y, bits=bits, hadamard=hadamard, eps=EPS)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(y.view(torch.int16), want.view(torch.int16)), name
        # twice in a row on the same stream: the second call overwrites the first one's intermediates
        y2 = torch.full((T, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        hbl.bitlinear_forward_small(x, packed, N, alphas, y2, bits=bits, hadamard=hadamard, eps=EPS)
        torch.cuda.synchronize()
        assert torch.equal(y2.view(torch.int16), want.view(torch.int16)), name


def test_no_alloc_forward_rejects_what_does_not_fit(hbl):
    site, x, packed, alphas = problem(hbl, "big", 65, 512, 64, True, 1, 7)
    y = torch.empty((65, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(hbl.HblError) as e:
        hbl.bitlinear_forward_small(x, packed, 64, alphas, y)
    assert e.value.status == hbl.E_SCRATCH
    with pytest.raises(hbl.HblError) as e:
        hbl.bitlinear_forward_small(x[:4, :384].contiguous(), packed, 64, alphas, y[:4].contiguous())
    assert e.value.status == hbl.E_SHAPE
    # an empty batch is a no-op
    hbl.bitlinear_forward_small(x[:0], packed, 64, alphas, y[:0])
