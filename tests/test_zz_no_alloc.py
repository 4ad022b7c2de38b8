"""kb_query_static (the entry point that allocates nothing) against kb_query, through the C ABI: two calls in a
row on the library's static scratch array, the second with a smaller input, bit for bit."""
import pytest
import torch

from paper_2602_14293_amd import kb as kbmod
from paper_2602_14293_amd import workloads as W

pytestmark = pytest.mark.gpu


def _both(w, masked):
    kb = kbmod.KnowledgeBase(w.d, kbmod.KB_BF16, w.N, tagged=True)
    kb.append(w.keys.cuda().contiguous(), None, w.tags.cuda())
    kb.normalize()
    q = w.queries.cuda().contiguous()
    qm = w.qmask.cuda() if masked else None
    want_i, want_s = kb.query(q, w.k, qm)
    got_i = torch.full((w.Q, w.k), -7, dtype=torch.int32, device="cuda")
    got_s = torch.full((w.Q, w.k), float("nan"), dtype=torch.float32, device="cuda")
    kb.query_static(q, w.k, qm, got_i, got_s)
    torch.cuda.synchronize()
    return kb, (want_i, want_s), (got_i, got_s)


def test_static_scratch_query_matches_kb_query_on_two_calls_in_a_row():
    big = W.filtered(seed=41, N=60000 + 19, d=512, Q=300, k=32, centers=32)         # two query blocks, ragged last tile
    small = W.filtered(seed=42, N=9000 + 5, d=512, Q=40, k=8, centers=16)           # a smaller input on the same scratch
    for w, masked in ((big, True), (small, False)):
        kb, want, got = _both(w, masked)
        assert torch.equal(want[0], got[0]), f"indices differ (N={w.N}, Q={w.Q})"
        assert torch.equal(want[1].view(torch.int32), got[1].view(torch.int32)), f"scores differ (N={w.N}, Q={w.Q})"
        assert (got[0][:, 0] >= 0).all()
        kb.close()


def test_static_scratch_query_rejects_what_does_not_fit():
    w = W.filtered(seed=43, N=4000, d=256, Q=8, k=8, centers=8)
    kb = kbmod.KnowledgeBase(w.d, kbmod.KB_BF16, w.N, tagged=True)
    kb.append(w.keys.cuda().contiguous(), None, w.tags.cuda())
    kb.normalize()
    Q, k = 20000, 128                                                                  # far beyond the array
    assert kbmod.lib().kb_query_plan_bytes(kb._h, kb.size, Q, k, 0) > (32 << 20)
    q = torch.zeros((Q, w.d), dtype=torch.bfloat16, device="cuda")
    out_i = torch.empty((Q, k), dtype=torch.int32, device="cuda")
    out_s = torch.empty((Q, k), dtype=torch.float32, device="cuda")
    with pytest.raises(kbmod.KBError) as e:
        kb.query_static(q, k, None, out_i, out_s)
    assert e.value.status == 7                                                         # KB_ERR_WORKSPACE
    kb.close()
