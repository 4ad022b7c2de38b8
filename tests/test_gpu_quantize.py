"""GPU parity of kb_quantize_rows (bit-exact codes and scales against the oracle) and of retrieval on what it
produces: fp8 queries against fp8 keys, checked on the codes and against the unquantised queries."""
import numpy as np
import pytest
import torch

from paper_2602_14293_amd import kb as kbmod
from paper_2602_14293_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def T():
    import kb_testlib

    return kb_testlib


def _check_rows(x: torch.Tensor, label: str):
    from oracle import kb_oracle

    codes, scale = kbmod.quantize_rows(x.cuda().contiguous())
    torch.cuda.synchronize()
    o_codes, o_scale = kb_oracle.quantize_rows(W.key_bits(x), kb_oracle.F32 if x.dtype == torch.float32 else kb_oracle.BF16)
    g_codes = codes.view(torch.uint8).cpu().numpy()
    assert np.array_equal(scale.cpu().numpy(), o_scale), f"{label}: scales differ"
    bad = np.argwhere(g_codes != o_codes)
    assert bad.size == 0, f"{label}: {len(bad)} codes differ, first at {bad[0]}: gpu {g_codes[tuple(bad[0])]:#x} oracle {o_codes[tuple(bad[0])]:#x}"
    return g_codes, o_scale


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n,d", [(1, 16), (5, 48), (777, 272), (300, 1024), (37, 2064), (9, 4112), (3, 16384)])
def test_codes_and_scales_are_bit_exact(dtype, n, d):
    g = torch.Generator().manual_seed(n * 100003 + d)
    x = torch.randn(n, d, generator=g) * torch.logspace(-8, 8, n)[:, None]
    x[n // 2] = 0                                                  # a zero row: scale 1, codes 0
    _check_rows(x.to(dtype), f"{dtype} n={n} d={d}")


def test_ties_saturation_and_tiny_rows():
    from oracle import kb_oracle

    vals = np.array([kb_oracle.decode_e4m3(c) for c in range(0x7F)])
    mids = ((vals[:-1] + vals[1:]) / 2).astype(np.float32)         # every tie, exactly representable
    row = np.zeros(512, dtype=np.float32)
    row[:126] = mids
    row[126:252] = -mids
    row[252:378] = np.nextafter(mids, np.float32(0))
    row[378:504] = np.nextafter(mids, np.float32(1e9))
    row[504] = 448.0                                               # the row maximum: scale is exactly 1
    row[505] = -0.0
    x = torch.from_numpy(np.stack([row, row * np.float32(2.0 ** -20), row * np.float32(2.0 ** 40), row * np.float32(2.0 ** -100)]))
    codes, scale = _check_rows(x, "ties")
    assert scale[0] == 1.0 and codes[0, 504] == 0x7E and codes[0, 505] == 0x80
    assert np.array_equal(codes[0], codes[1]) and np.array_equal(codes[0], codes[2]) and np.array_equal(codes[0], codes[3])


def test_large_matrix_sampled_rows():
    # the size of a whole query batch / an append block: every row checked for the scale, sampled rows for the codes
    from oracle import kb_oracle

    g = torch.Generator().manual_seed(99)
    x = torch.randn(20000, 768, generator=g).to(torch.bfloat16)
    codes, scale = kbmod.quantize_rows(x.cuda())
    torch.cuda.synchronize()
    pick = torch.randperm(20000, generator=g)[:500]
    o_codes, o_scale = kb_oracle.quantize_rows(W.key_bits(x[pick]), kb_oracle.BF16)
    assert np.array_equal(codes[pick.cuda()].view(torch.uint8).cpu().numpy(), o_codes)
    assert np.array_equal(scale[pick.cuda()].cpu().numpy(), o_scale)
    amax = x.float().abs().amax(dim=1)
    assert torch.equal(scale.cpu(), amax / 448.0)


def test_no_scale_wanted():
    x = torch.randn(64, 128, generator=torch.Generator().manual_seed(1))
    a, s = kbmod.quantize_rows(x.cuda(), want_scale=True)
    b, none = kbmod.quantize_rows(x.cuda(), want_scale=False)
    torch.cuda.synchronize()
    assert none is None and torch.equal(a.view(torch.uint8), b.view(torch.uint8))


@pytest.mark.parametrize("seed", [0, 1])
def test_quantised_queries_against_quantised_keys(T, seed):
    """bf16 rows and bf16 queries, both quantised on the GPU, retrieved through the fp8 x fp8 path.  Checked
    (a) on the codes: the oracle scores the same stored bits, tight tolerance; (b) against the oracle on the
    UNQUANTISED queries: rounding a query to e4m3 (relative step 2^-3, error uniform within +-2^-4) moves a cosine
    by about 0.036 / sqrt(d) rms, far inside the 2e-2 tolerance of fp8 storage, so the index sets agree up to near-ties."""
    from oracle import compare, kb_oracle

    src = W.clustered(seed=seed, N=30000, d=768, Q=200, k=32, centers=64)          # bf16 keys and queries
    k8, kscale = kbmod.quantize_rows(src.keys.cuda())
    q8, _ = kbmod.quantize_rows(src.queries.cuda(), want_scale=False)
    torch.cuda.synchronize()
    w = W.Workload("quantised", k8.cpu(), q8.cpu(), src.k, scale=kscale.cpu(), seed=seed)
    rep, cnt, (gi, gs) = T.run_and_check(w, label=f"quantised seed {seed}")        # (a)
    assert rep.queries == 200
    full = kb_oracle.score_matrix(W.key_bits(w.keys), kb_oracle.FP8_E4M3, W.key_bits(src.queries), kb_oracle.BF16,
                                  row_scale=w.scale.numpy())
    rep2 = compare.check(gi, gs, full, src.k, 2e-2, label="fp8 queries against the bf16-query oracle")   # (b)
    assert rep2.max_score_err < 0.036 / np.sqrt(768) * 6, rep2.max_score_err
