"""GPU parity of knowledge-base maintenance: revised gains, removed entries in every query path, compaction."""
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


# ---------------- kb_update_gain -----------------------------------------------------------------

@pytest.mark.parametrize("alpha", [0.0, 0.25, 0.9, 1.0])
def test_gain_update_matches_the_oracle(alpha):
    from oracle import kb_oracle

    rng = np.random.default_rng(int(alpha * 100))
    n, m = 50000, 7000
    gain = rng.uniform(0.1, 8.0, n).astype(np.float32)
    idx = rng.choice(n, size=m, replace=False).astype(np.int32)
    idx[::50] = -1                                                 # the padding of a result list is skipped
    idx[1::97] = n + 5                                             # as is anything else out of range
    val = rng.uniform(0.0, 10.0, m).astype(np.float32)
    g = torch.from_numpy(gain).cuda()
    kbmod.update_gain(g, torch.from_numpy(idx).cuda(), torch.from_numpy(val).cuda(), alpha)
    torch.cuda.synchronize()
    want = kb_oracle.update_gain(gain, idx, val, alpha)
    got = g.cpu().numpy().astype(np.float64)
    # fp32: one rounded subtraction and one fma, each within 2^-24 relative of values below 10
    assert np.abs(got - want).max() <= 2 * 10.0 * 2.0 ** -24
    touched = np.zeros(n, dtype=bool)
    touched[idx[(idx >= 0) & (idx < n)]] = True
    assert np.array_equal(got[~touched], gain[~touched].astype(np.float64))
    if alpha == 1.0:
        ok = (idx >= 0) & (idx < n)
        assert np.array_equal(g.cpu().numpy()[idx[ok]], val[ok])


def test_updated_gains_steer_the_weighted_selection(T):
    """Entries whose gain has been raised are drawn accordingly: the draw with revised gains against the oracle's draw
    with the oracle's revised gains (both sides revise on their own; keys agree within the key tolerance)."""
    from oracle import compare, kb_oracle

    w = W.filtered(seed=31, N=9000, d=256, Q=48, k=16, centers=32)
    kb = T.build_kb(w)
    rng = np.random.default_rng(4)
    gain = rng.uniform(0.5, 2.0, w.N).astype(np.float32)
    idx = rng.choice(w.N, size=600, replace=False).astype(np.int32)
    val = rng.uniform(200.0, 400.0, 600).astype(np.float32)
    g = torch.from_numpy(gain).cuda()
    kbmod.update_gain(g, torch.from_numpy(idx).cuda(), torch.from_numpy(val).cuda(), 0.5)
    gi, gk = kb.query_sampled(w.queries.cuda(), w.k, g, 0.5, 77, w.qmask.cuda())
    torch.cuda.synchronize()
    g_oracle = kb_oracle.update_gain(gain, idx, val, 0.5).astype(np.float32)
    keys = kb_oracle.selection_keys(T.oracle_scores(w), g_oracle, 0.5, 77)
    rep = compare.check(gi.cpu().numpy(), gk.cpu().numpy(), keys, w.k, 2e-4, tags=W.word_bits(w.tags), qmask=W.word_bits(w.qmask),
                        label="draw with revised gains")
    assert rep.queries == 48
    raised = np.isin(gi.cpu().numpy(), idx).mean()
    assert raised > 0.6                                             # 6.7 % of the entries carry about 90 % of the weight now
    kb.close()


# ---------------- kb_remove ----------------------------------------------------------------------

def _removal_set(T, w, rng, use_mask, frac=0.1, best=5):
    """Indices to remove: the oracle's best few of every query (so results must change), a random share, junk."""
    from oracle import kb_oracle

    full = T.oracle_scores(w)
    removed = rng.random(w.N) < frac
    tags = W.word_bits(w.tags) if use_mask else None
    for r in range(w.Q):
        qm = W.word_bits(w.qmask)[r] if use_mask else None
        idx, _, n = kb_oracle.select(full[r], best, tags=tags, qmask=qm)
        removed[idx[:min(n, best)]] = True
    idx = np.flatnonzero(removed).astype(np.int32)
    sent = np.concatenate([idx, idx[:7], np.array([-1, -5, w.N, w.N + 100], dtype=np.int32)])   # repeats and junk are harmless
    rng.shuffle(sent)
    return removed, sent


@pytest.mark.parametrize("kind,N,d,Q,k", [("f32", 5000, 128, 20, 16), ("bf16", 20077, 256, 64, 32), ("bf16", 17000, 512, 300, 32),
                                          ("fp8", 9000, 512, 40, 16), ("fp8", 17077, 512, 300, 64)])
def test_removed_entries_never_come_back(T, kind, N, d, Q, k):
    rng = np.random.default_rng(N + Q)
    if kind == "f32":
        w = W.tiny(seed=N, N=N, d=d, Q=Q, k=k)
    elif kind == "bf16":
        w = W.filtered(seed=N, N=N, d=d, Q=Q, k=k, centers=32)
    else:
        w = W.compressed(seed=N, N=N, d=d, Q=Q, k=k, centers=32)
    use_mask = w.qmask is not None
    kb = T.build_kb(w)
    before_i, _ = T.gpu_query(kb, w, use_mask)
    removed, sent = _removal_set(T, w, rng, use_mask)
    kb.remove(torch.from_numpy(sent).cuda())
    assert kb.size == w.N                                           # indices are stable
    gi, gs = T.gpu_query(kb, w, use_mask)
    rep = T.check_against_oracle(w, gi, gs, use_mask, label=f"removed {kind} N={N} Q={Q}", removed=removed)
    assert rep.queries == Q and not removed[gi[gi >= 0]].any()
    assert (before_i != gi).any()                                   # the best entries of every query were among the removed
    if use_mask:                                                    # and without the tag filter too
        gi, gs = T.gpu_query(kb, w, False)
        T.check_against_oracle(w, gi, gs, False, label=f"removed {kind} unmasked", removed=removed)
    kb.close()


def test_removal_down_to_a_handful_pads_and_takes_the_exhaustive_path(T):
    w = W.filtered(seed=8, N=3000, d=256, Q=12, k=8, centers=4)
    kb = T.build_kb(w)
    removed = np.ones(w.N, dtype=bool)
    removed[[5, 1700, 2999]] = False
    kb.remove(torch.from_numpy(np.flatnonzero(removed).astype(np.int32)).cuda())
    gi, gs = T.gpu_query(kb, w, False)
    T.check_against_oracle(w, gi, gs, False, label="three left", removed=removed)
    assert (gi[:, 3:] == -1).all() and set(gi[:, :3].ravel().tolist()) == {5, 1700, 2999}
    kb.remove(torch.tensor([5, 1700, 2999], dtype=torch.int32).cuda())
    gi, gs = T.gpu_query(kb, w, False)
    assert (gi == -1).all() and np.isneginf(gs).all()
    kb.close()


def test_removed_zero_row_and_live_zero_row(T):
    keys = torch.randn(100, 64, generator=torch.Generator().manual_seed(2))
    keys[10] = 0
    keys[20] = 0
    q = -keys[:3].clone()
    w = W.Workload("zeros", keys, q, 100)
    kb = T.build_kb(w)
    kb.remove(torch.tensor([10], dtype=torch.int32).cuda())        # 1/|k| = 0 becomes -0: still marked
    removed = np.zeros(100, dtype=bool)
    removed[10] = True
    gi, gs = T.gpu_query(kb, w, False)
    T.check_against_oracle(w, gi, gs, False, label="zero rows", removed=removed)
    assert (gi == 20).any(axis=1).all() and not (gi == 10).any() and (gi[:, -1] == -1).all()
    kb.close()


def test_removal_applies_to_the_weighted_selection(T):
    from oracle import compare, kb_oracle

    w = W.filtered(seed=41, N=9000, d=256, Q=40, k=16, centers=32)
    kb = T.build_kb(w)
    rng = np.random.default_rng(9)
    removed, sent = _removal_set(T, w, rng, True, frac=0.3)
    kb.remove(torch.from_numpy(sent).cuda())
    gain = rng.uniform(0.5, 2.0, w.N).astype(np.float32)
    gi, gk = kb.query_sampled(w.queries.cuda(), w.k, torch.from_numpy(gain).cuda(), 0.2, 5, w.qmask.cuda())
    torch.cuda.synchronize()
    keys = kb_oracle.without_removed(kb_oracle.selection_keys(T.oracle_scores(w), gain, 0.2, 5), removed)
    compare.check(gi.cpu().numpy(), gk.cpu().numpy(), keys, w.k, 2e-4, tags=W.word_bits(w.tags), qmask=W.word_bits(w.qmask),
                  label="draw after removal")
    assert not removed[gi.cpu().numpy()].any()
    kb.close()


def test_remove_needs_normalised_rows(T):
    w = W.tiny(seed=1, N=300, d=64, Q=2, k=4)
    kb = kbmod.KnowledgeBase(w.d, kbmod.KB_F32, 400)
    kb.append(w.keys.cuda())
    with pytest.raises(kbmod.KBError) as e:
        kb.remove(torch.tensor([1], dtype=torch.int32).cuda())
    assert e.value.status == 5
    kb.close()


# ---------------- kb_compact ---------------------------------------------------------------------

@pytest.mark.parametrize("kind,N,d", [("bf16", 20077, 256), ("fp8", 9100, 512), ("f32", 1000, 96), ("bf16", 130, 64)])
def test_compaction_moves_the_live_entries_bit_for_bit(T, kind, N, d):
    from oracle import kb_oracle

    rng = np.random.default_rng(N)
    Q, k = 24, 16
    if kind == "f32":
        w = W.tiny(seed=N, N=N, d=d, Q=Q, k=k)
    elif kind == "bf16":
        w = W.filtered(seed=N, N=N, d=d, Q=Q, k=k, centers=16)
    else:
        w = W.compressed(seed=N, N=N, d=d, Q=Q, k=k, centers=16)
    use_mask = w.qmask is not None
    src = T.build_kb(w)
    removed, sent = _removal_set(T, w, rng, use_mask, frac=0.35)
    src.remove(torch.from_numpy(sent).cuda())
    gain = rng.uniform(0.5, 2.0, w.N).astype(np.float32)
    arrays = [W.key_bits(w.keys), gain] + ([W.word_bits(w.tags)] if w.tags is not None else []) + ([w.scale.numpy()] if w.scale is not None else [])
    want_map, want = kb_oracle.compact(removed, *arrays)
    n_live = int((~removed).sum())

    small = kbmod.KnowledgeBase(w.d, T.CODE[w.keys.dtype], n_live - 1, tagged=w.tags is not None)
    with pytest.raises(kbmod.KBError) as e:                        # too small: refused, nothing written
        src.compact_into(small)
    assert e.value.status == 4 and small.size == 0
    small.close()

    dst = kbmod.KnowledgeBase(w.d, T.CODE[w.keys.dtype], n_live + 3, tagged=w.tags is not None)
    live, index_map, gain_dst = src.compact_into(dst, gain=torch.from_numpy(gain).cuda())
    torch.cuda.synchronize()
    assert live == n_live and dst.size == n_live and src.size == w.N
    assert np.array_equal(index_map.cpu().numpy(), want_map)
    assert np.array_equal(W.key_bits(dst.keys[:live].cpu()), want[0])
    assert np.array_equal(gain_dst.cpu().numpy(), want[1])
    nxt = 2
    if w.tags is not None:
        assert np.array_equal(W.word_bits(dst.tags[:live].cpu()), want[nxt])
        nxt += 1
    if w.scale is not None:
        assert np.array_equal(dst.scale[:live].cpu().numpy(), want[nxt])
    # retrieval on the compacted store against the oracle on the oracle's compacted arrays
    w2 = W.Workload("compacted", torch.from_numpy(want[0]).view(w.keys.dtype) if kind != "f32" else torch.from_numpy(want[0]),
                    w.queries, w.k, scale=None if w.scale is None else torch.from_numpy(want[nxt]),
                    tags=None if w.tags is None else torch.from_numpy(want[2].view(np.int64)), qmask=w.qmask)
    gi, gs = T.gpu_query(dst, w2, use_mask)
    T.check_against_oracle(w2, gi, gs, use_mask, label=f"compacted {kind} N={N}")
    # and it is the same answer as on the store with removed entries, under the index map
    gi0, gs0 = T.gpu_query(src, w, use_mask)
    back = np.flatnonzero(~removed)
    assert np.array_equal(np.where(gi >= 0, back[np.maximum(gi, 0)], -1), gi0) and np.array_equal(gs, gs0)
    src.close()
    dst.close()


def test_compaction_with_nothing_or_everything_removed(T):
    w = W.filtered(seed=3, N=700, d=128, Q=4, k=8, centers=4)
    src = T.build_kb(w)
    dst = kbmod.KnowledgeBase(w.d, kbmod.KB_BF16, 700, tagged=True)
    live, index_map, _ = src.compact_into(dst)
    torch.cuda.synchronize()
    assert live == 700 and index_map.cpu().tolist() == list(range(700))
    assert torch.equal(dst.keys.view(torch.int16).cpu(), w.keys.view(torch.int16)) and torch.equal(dst.tags.cpu(), w.tags)
    src.remove(torch.arange(700, dtype=torch.int32).cuda())
    dst2 = kbmod.KnowledgeBase(w.d, kbmod.KB_BF16, 10, tagged=True)
    live, index_map, _ = src.compact_into(dst2)
    assert live == 0 and dst2.size == 0 and (index_map.cpu() == -1).all()
    gi, gs = dst2.query(w.queries.cuda(), 8)
    torch.cuda.synchronize()
    assert (gi.cpu() == -1).all()
    for h in (src, dst, dst2):
        h.close()
