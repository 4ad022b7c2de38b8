"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle on the same seeded inputs."""
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


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_tiny_f32_full_config(T, seed):
    w = W.tiny(seed=seed)                      # N=4096 d=256 Q=8 k=8 fp32
    rep, cnt, _ = T.run_and_check(w, label=f"tiny seed {seed}")
    assert rep.queries == 8 and cnt["exhaustive_queries"] == 0


@pytest.mark.parametrize("N,d,Q,k", [(1000, 96, 5, 7), (129, 32, 1, 1), (50, 64, 3, 64), (4097, 128, 40, 33), (2500, 64, 130, 5)])
def test_f32_shapes(T, N, d, Q, k):
    w = W.tiny(seed=N + Q, N=N, d=d, Q=Q, k=k)
    T.run_and_check(w, label=f"f32 N={N} d={d} Q={Q} k={k}")


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_clustered_bf16_reduced(T, seed):
    w = W.clustered(seed=seed, N=20000 + 37 * seed, d=768, Q=64, k=16, centers=64)
    rep, cnt, _ = T.run_and_check(w, label=f"clustered seed {seed}")
    assert cnt["sample_keys"] > 0 and cnt["exhaustive_queries"] == 0


@pytest.mark.parametrize("N,d,Q,k", [(5000, 192, 31, 9), (3001, 64, 70, 16), (9000, 256, 300, 32), (700, 128, 257, 128), (64, 64, 2, 3)])
def test_bf16_shapes(T, N, d, Q, k):
    w = W.clustered(seed=N, N=N, d=d, Q=Q, k=k, centers=16)
    T.run_and_check(w, label=f"bf16 N={N} d={d} Q={Q} k={k}")


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_filtered_bf16_reduced(T, seed):
    w = W.filtered(seed=seed, N=30000, d=1024, Q=256, k=32, centers=64)
    rep, cnt, _ = T.run_and_check(w, label=f"filtered seed {seed}")
    assert rep.queries == 256


@pytest.mark.parametrize("config", [3, 12, 16, 17, 18, 19])
def test_every_large_batch_scan_kernel(T, config):
    """Each scan kernel that handles 256-query blocks (tiled, software-pipelined, full-line) gives
    the same oracle-checked result; ragged last tile, 300 queries = two query blocks, masked."""
    w = W.filtered(seed=7, N=20000 + 131, d=512, Q=300, k=32, centers=32)
    rep, cnt, _ = T.run_and_check(w, label=f"scan config {config}", tuning={"scan_config": config})
    assert rep.queries == 300 and cnt["exhaustive_queries"] == 0


@pytest.mark.parametrize("config", [17, 18, 19])
def test_several_items_and_query_blocks_per_workgroup(T, config):
    """More (key tile, query block) items than workgroups AND more than one query block: a workgroup's stream crosses
    item boundaries where the query block changes (the per-query side data in LDS is reloaded there), with the
    shortest rows the pipelined kernels take (four 128-byte chunks) and a ragged last tile."""
    w = W.filtered(seed=21, N=50000 + 57, d=256, Q=300, k=32, centers=32)
    rep, cnt, _ = T.run_and_check(w, label=f"many items, scan config {config}", tuning={"scan_config": config})
    assert rep.queries == 300 and cnt["exhaustive_queries"] == 0 and cnt["scan_workgroups"] == 256


@pytest.mark.parametrize("config,Q", [(18, 200), (19, 100)])
def test_full_line_kernels_without_mask_and_with_removed_rows(T, config, Q):
    """The full-line kernels on unmasked queries (no tag side data is loaded) with removed entries in the store."""
    import numpy as np

    w = W.clustered(seed=23, N=30000 + 11, d=320, Q=Q, k=16, centers=16)
    kb = T.build_kb(w)
    kb.set_tuning("scan_config", config)
    before_i, _ = T.gpu_query(kb, w)
    removed = np.zeros(w.N, dtype=bool)
    removed[np.unique(before_i[:, :4])] = True                      # the best four of every query, and every 97th row
    removed[5::97] = True
    kb.remove(torch.from_numpy(np.flatnonzero(removed).astype(np.int32)).cuda())
    gi, gs = T.gpu_query(kb, w)
    rep = T.check_against_oracle(w, gi, gs, label=f"unmasked, removed rows, scan config {config}", removed=removed)
    assert rep.queries == Q and not removed[gi[gi >= 0]].any() and kb.counters()["exhaustive_queries"] == 0
    kb.close()


@pytest.mark.parametrize("seed", [0, 1])
def test_sparse_filter_exercises_padding(T, seed):
    w = W.filtered(seed=seed, N=12000, d=256, Q=96, k=32, centers=16, p_tag=0.003, single_bit_qmask=True)
    rep, cnt, (gi, gs) = T.run_and_check(w, label=f"sparse filter seed {seed}")
    assert (gi < 0).any()                       # some queries have fewer than k qualifying entries


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_compressed_fp8_reduced(T, seed):
    w = W.compressed(seed=seed, N=24000, d=768, Q=100, k=64, centers=64)
    T.run_and_check(w, label=f"compressed seed {seed}")


@pytest.mark.parametrize("config", [3, 4])
def test_every_large_batch_fp8_scan_kernel(T, config):
    w = W.compressed(seed=11, N=17000 + 77, d=512, Q=300, k=64, centers=32)
    rep, cnt, _ = T.run_and_check(w, label=f"fp8 scan config {config}", tuning={"scan_config": config})
    assert rep.queries == 300 and cnt["exhaustive_queries"] == 0


@pytest.mark.parametrize("config", [5, 20])
def test_every_fp8_query_scan_kernel(T, config):
    """Both kernels built on the fp8 matrix instruction (64-byte and 128-byte row pieces): several items and query
    blocks per workgroup, ragged last tile, checked against the oracle on the same codes."""
    w = W.compressed(seed=29, N=50000 + 57, d=512, Q=600, k=32, centers=32, fp8_queries=True)
    rep, cnt, _ = T.run_and_check(w, label=f"fp8 x fp8 scan config {config}", tuning={"scan_config": config})
    assert rep.queries == 600 and cnt["exhaustive_queries"] == 0 and cnt["scan_workgroups"] == 256


@pytest.mark.parametrize("config,Q", [(6, 50), (7, 130), (8, 600)])
def test_every_tiled_fp8_query_scan_kernel(T, config, Q):
    """The tiled kernel on the fp8 matrix instruction (query blocks of 64, 128 and 256), forced for a batch that spans
    several query blocks: ragged last tile, ragged last block."""
    w = W.compressed(seed=31, N=30000 + 41, d=512, Q=Q, k=32, centers=32, fp8_queries=True)
    rep, cnt, _ = T.run_and_check(w, label=f"fp8 x fp8 tiled scan config {config}", tuning={"scan_config": config})
    assert rep.queries == Q and cnt["exhaustive_queries"] == 0


@pytest.mark.parametrize("N,d,Q,k", [(3000, 256, 33, 20), (130, 64, 1, 1), (5000, 128, 260, 7), (9000, 256, 260, 16)])
def test_fp8_shapes(T, N, d, Q, k):
    w = W.compressed(seed=N, N=N, d=d, Q=Q, k=k, centers=8)
    T.run_and_check(w, label=f"fp8 N={N} d={d} Q={Q} k={k}")


@pytest.mark.parametrize("N,d,Q,k", [(24000, 768, 100, 64), (17077, 512, 300, 64), (3000, 384, 33, 20), (130, 448, 1, 1),
                                     (70000, 1024, 700, 128), (3000, 256, 33, 20), (130, 64, 1, 1), (5000, 128, 260, 7),
                                     (40000, 192, 100, 16), (33000, 320, 20, 8)])
def test_fp8_queries_on_fp8_keys(T, N, d, Q, k):
    # both operands in e4m3: scored by the fp8 matrix instruction, checked against the oracle on the same codes
    w = W.compressed(seed=N + 1, N=N, d=d, Q=Q, k=k, centers=32, fp8_queries=True)
    assert w.queries.dtype == torch.float8_e4m3fn
    rep, cnt, (gi, gs) = T.run_and_check(w, label=f"fp8 x fp8 N={N} d={d} Q={Q} k={k}")
    assert rep.queries == Q


def test_fp8_queries_exhaustive_path_and_short_rows(T):
    # few keys: every query is resolved by the exhaustive path, which must score exactly like the scan
    w = W.compressed(seed=5, N=700, d=512, Q=40, k=16, centers=8, fp8_queries=True)
    rep, cnt, _ = T.run_and_check(w, label="fp8 x fp8 small")
    # rows shorter than the pipelined kernels' rings go to the tiled kernel
    w2 = W.compressed(seed=6, N=500, d=256, Q=4, k=4, centers=8, fp8_queries=True)
    T.run_and_check(w2, label="fp8 x fp8 small, short rows")


def test_all_e4m3_codes_decode_like_the_oracle(T):
    # keys whose rows run through every finite e4m3 code; one-hot queries read single elements back
    codes = torch.tensor([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=torch.uint8)
    d = 256
    rows = torch.zeros(8, d, dtype=torch.uint8)
    rows[0, :254] = codes
    rows[1, :254] = codes.flip(0)
    for r in range(2, 8):
        rows[r] = torch.roll(rows[0], 37 * r)
    keys = rows.view(torch.float8_e4m3fn)
    scale = torch.ones(8)
    queries = torch.randn(16, d, generator=torch.Generator().manual_seed(0)).to(torch.bfloat16)
    w = W.Workload("codes", keys, queries, k=8, scale=scale)
    T.run_and_check(w, label="all e4m3 codes")


def test_mask_edge_cases(T):
    w = W.filtered(seed=5, N=3000, d=64, Q=8, k=4, centers=4)
    w.qmask[0] = 0                                      # zero mask word: nothing qualifies
    w.tags[:100] = 0                                    # untagged entries never qualify under a mask
    w.qmask[1] = -1                                     # all bits
    kb = T.build_kb(w)
    gi, gs = T.gpu_query(kb, w)
    assert (gi[0] == -1).all() and np.isneginf(gs[0]).all()
    assert (gi[1:] >= 100).all()
    T.check_against_oracle(w, gi, gs, label="mask edges")
    gi2, gs2 = T.gpu_query(kb, w, use_mask=False)       # NULL mask on a tagged KB: no filtering
    T.check_against_oracle(w, gi2, gs2, use_mask=False, label="null mask")
    kb.close()


def test_duplicate_rows_tie_break_is_exact(T):
    # identical rows at indices spread over tile and workgroup boundaries must get identical scores and
    # come back in ascending index order
    w = W.clustered(seed=9, N=6000, d=128, Q=4, k=12, centers=4)
    dup = [3, 127, 128, 129, 255, 256, 1000, 2047, 2048, 4095, 4096, 5999]
    src = w.queries[0].clone()
    w.keys[dup] = src
    kb = T.build_kb(w)
    gi, gs = T.gpu_query(kb, w)
    assert gi[0].tolist() == dup
    assert len(set(gs[0].tolist())) == 1 and abs(gs[0][0] - 1.0) <= 1e-6
    T.check_against_oracle(w, gi, gs, label="duplicates")
    kb.close()


def test_self_query_and_permutation(T):
    w = W.clustered(seed=11, N=4000, d=256, Q=16, k=8, centers=8)
    pick = torch.arange(16) * 250 + 3
    w.queries = w.keys[pick].clone()
    kb = T.build_kb(w)
    gi, gs = T.gpu_query(kb, w)
    assert gi[:, 0].tolist() == pick.tolist() and np.abs(gs[:, 0] - 1.0).max() <= 1e-6
    perm = torch.randperm(4000, generator=torch.Generator().manual_seed(1))
    w2 = W.Workload("perm", w.keys[perm].contiguous(), w.queries, w.k)
    kb2 = T.build_kb(w2)
    gi2, gs2 = T.gpu_query(kb2, w2)
    assert np.array_equal(perm.numpy()[gi2], gi) and np.array_equal(gs2, gs)
    kb.close(); kb2.close()


def test_zero_rows_and_zero_query(T):
    w = W.tiny(seed=13, N=600, d=64, Q=4, k=10)
    w.keys[5] = 0
    w.keys[300] = 0
    w.queries[2] = 0
    rep, cnt, (gi, gs) = T.run_and_check(w, label="zeros")
    assert gi[2].tolist() == list(range(10)) and (gs[2] == 0).all()      # zero query: all scores 0, lowest indices
    assert not np.isnan(gs).any()


def test_exhaustive_path_on_degenerate_data(T):
    # every key identical: every score ties, the threshold cannot prune, candidate lists overflow and the
    # exhaustive per-query path must still return the k lowest indices
    w = W.clustered(seed=15, N=20000, d=64, Q=3, k=5, centers=2)
    w.keys[:] = w.keys[0]
    rep, cnt, (gi, gs) = T.run_and_check(w, label="all keys equal")
    assert gi.tolist() == [[0, 1, 2, 3, 4]] * 3


def test_append_normalize_query_rounds(T):
    # growing KB: appends that straddle tile boundaries; each round checked against an oracle on the KB so far
    base = W.filtered(seed=21, N=3000, d=128, Q=8, k=16, centers=8)
    kb = kbmod.KnowledgeBase(128, kbmod.KB_BF16, 6200, tagged=True)
    keys_all, tags_all = base.keys.clone(), base.tags.clone()
    assert kb.append(base.keys.cuda(), None, base.tags.cuda()) == 0
    with pytest.raises(kbmod.KBError) as e:
        kb.query(base.queries.cuda(), 16, base.qmask.cuda())
    assert e.value.status == 5                                         # KB_ERR_NOT_NORMALIZED
    kb.normalize()
    kb.normalize()                                                     # idempotent
    inv_before = kb.inv_norm[:3000].clone()
    for r in range(4):
        extra = W.filtered(seed=100 + r, N=777, d=128, Q=8, k=16, centers=8)
        first = kb.append(extra.keys.cuda(), None, extra.tags.cuda())
        assert first == keys_all.shape[0]
        kb.normalize()
        keys_all = torch.cat([keys_all, extra.keys]); tags_all = torch.cat([tags_all, extra.tags])
        w = W.Workload("grow", keys_all, extra.queries, 16, tags=tags_all, qmask=extra.qmask)
        gi, gs = T.gpu_query(kb, w)
        T.check_against_oracle(w, gi, gs, label=f"growing round {r}")
        assert kb.size == keys_all.shape[0]
    assert torch.equal(kb.inv_norm[:3000], inv_before)                 # old rows untouched
    with pytest.raises(kbmod.KBError) as e:
        kb.append(base.keys.cuda(), None, base.tags.cuda())
    assert e.value.status == 4                                         # KB_ERR_CAPACITY
    kb.close()


def test_run_to_run_determinism(T):
    w = W.filtered(seed=31, N=25000, d=256, Q=200, k=32, centers=32)
    kb = T.build_kb(w)
    a = T.gpu_query(kb, w)
    for _ in range(3):
        b = T.gpu_query(kb, w)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1].view(np.uint32), b[1].view(np.uint32))
    kb.close()


def test_empty_kb_returns_padding(T):
    kb = kbmod.KnowledgeBase(64, kbmod.KB_BF16, 16)
    q = torch.randn(3, 64).to(torch.bfloat16).cuda()
    gi, gs = kb.query(q, 4)
    torch.cuda.synchronize()
    assert (gi.cpu().numpy() == -1).all() and np.isneginf(gs.cpu().numpy()).all()
    kb.close()


def test_query_replays_from_a_captured_graph(T):
    """kb_query allocates nothing, never synchronises and records no memset, so it can be captured in a HIP graph.
    Every replay (with eager work and synchronisations in between, and with new query contents in the captured
    buffers) must give the bits of an eager call on the same inputs."""
    w = W.filtered(seed=5, N=30000 + 19, d=512, Q=200, k=24, centers=32)
    w2 = W.filtered(seed=6, N=30000 + 19, d=512, Q=200, k=24, centers=32)
    kb = T.build_kb(w)
    dev = kb.keys.device
    queries, qmask = w.queries.to(dev).contiguous(), w.qmask.to(dev).contiguous()
    out_i = torch.empty((w.Q, w.k), dtype=torch.int32, device=dev)
    out_s = torch.empty((w.Q, w.k), dtype=torch.float32, device=dev)
    kb.query(queries, w.k, qmask, out_i, out_s)             # warm-up: one-time kernel attributes are set outside the capture
    torch.cuda.synchronize()
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        kb.query(queries, w.k, qmask, out_i, out_s)
    torch.cuda.synchronize()
    for rep in range(4):
        src = w if rep % 2 == 0 else w2
        queries.copy_(src.queries.to(dev))
        qmask.copy_(src.qmask.to(dev))
        ref_i, ref_s = kb.query(queries, w.k, qmask)        # eager, into fresh outputs
        torch.cuda.synchronize()
        out_i.fill_(-7)
        out_s.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_i, ref_i) and torch.equal(out_s, ref_s), f"replay {rep} differs from the eager call"
    mixed = W.Workload("graph replay", w.keys, w2.queries, w.k, tags=w.tags, qmask=w2.qmask)     # the last replay's inputs
    T.check_against_oracle(mixed, out_i.cpu().numpy(), out_s.cpu().numpy(), label="graph replay")
    kb.close()


def test_scan_timing_counts_the_launches_it_times(T):
    """kb_profile_begin / kb_profile_end: every scan launch is timed by default, every n-th (the middle one of each run
    of n) with the "profile_stride" knob, never more than max_calls; timing changes no result."""
    w = W.filtered(seed=9, N=40000 + 7, d=512, Q=200, k=16, centers=32)
    kb = T.build_kb(w)
    dev = kb.keys.device
    queries, qmask = w.queries.to(dev).contiguous(), w.qmask.to(dev).contiguous()
    ref_i, ref_s = kb.query(queries, w.k, qmask)
    kb.profile_begin(16)
    for _ in range(10):
        gi, gs = kb.query(queries, w.k, qmask)
    ms, n = kb.profile_end()
    assert n == 10 and 0.0 < ms < 100.0 and torch.equal(gi, ref_i) and torch.equal(gs, ref_s)
    kb.set_tuning("profile_stride", 4)
    kb.profile_begin(16)
    for _ in range(10):
        gi, gs = kb.query(queries, w.k, qmask)
    ms4, n4 = kb.profile_end()
    assert n4 == 2 and 0.0 < ms4 < ms and torch.equal(gi, ref_i)         # launches 2 and 6 of 0..9
    kb.profile_begin(1)
    for _ in range(10):
        kb.query(queries, w.k, qmask)
    assert kb.profile_end()[1] == 1
    kb.set_tuning("profile_stride", 0)
    kb.profile_begin(4)
    for _ in range(3):
        kb.query(queries, w.k, qmask)
    assert kb.profile_end()[1] == 3
    kb.close()
