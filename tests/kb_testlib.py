"""Shared helpers of the GPU parity tests: run the HIP path and the fp64 oracle on the same stored bits."""
from __future__ import annotations

import numpy as np
import torch

from oracle import compare, kb_oracle
from paper_2602_14293_amd import kb as kbmod
from paper_2602_14293_amd import workloads as W

# Absolute score tolerances: fp32 keys 1e-5, bf16 2e-3, fp8 2e-2.  The oracle reads the same stored bits as
# the GPU, so the observed error is fp32-accumulation level (about 1e-6) for every dtype.  Every result is
# therefore judged by the whole acceptance rule (scores, membership, exact index set, order) a second time at
# TIGHT: at the dtype tolerance the k-th/(k+1)-th gap of these dense workloads (about 3e-4) is below tau for
# nearly every query, and a result that lost its k-th entry to the (k+1)-th would be accepted.
TAU = {kbmod.KB_F32: 1e-5, kbmod.KB_BF16: 2e-3, kbmod.KB_FP8_E4M3: 2e-2}
TIGHT = 1e-5
# fp8 queries go through the fp8 matrix instruction, which sums the 64 exact products of a chunk in hardware with
# less than fp32 precision per addend (measured: about 1e-5 of |q||k| per instruction on Gaussian rows)
TIGHT_FP8_QUERIES = 1e-4
ORACLE_DTYPE = {kbmod.KB_F32: kb_oracle.F32, kbmod.KB_BF16: kb_oracle.BF16, kbmod.KB_FP8_E4M3: kb_oracle.FP8_E4M3}
CODE = {torch.float32: kbmod.KB_F32, torch.bfloat16: kbmod.KB_BF16, torch.float8_e4m3fn: kbmod.KB_FP8_E4M3}


def build_kb(w: W.Workload, capacity=None, tagged=None) -> kbmod.KnowledgeBase:
    code = CODE[w.keys.dtype]
    tagged = (w.tags is not None) if tagged is None else tagged
    kb = kbmod.KnowledgeBase(w.d, code, capacity or max(w.N, 1), tagged=tagged)
    if w.N:
        kb.append(w.keys.cuda().contiguous(), None if w.scale is None else w.scale.cuda(),
                  None if not tagged else w.tags.cuda())
        kb.normalize()
    return kb


def gpu_query(kb, w: W.Workload, use_mask=True):
    qm = w.qmask.cuda() if (use_mask and w.qmask is not None) else None
    idx, sc = kb.query(w.queries.cuda().contiguous(), w.k, qm)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), sc.cpu().numpy()


def oracle_scores(w: W.Workload, rows=None):
    """fp64 score matrix of the stored bits (optionally for a subset of query rows)."""
    code = CODE[w.keys.dtype]
    q = w.queries if rows is None else w.queries[rows]
    qd = ORACLE_DTYPE[CODE[q.dtype]]
    return kb_oracle.score_matrix(W.key_bits(w.keys), ORACLE_DTYPE[code], W.key_bits(q), qd,
                                  row_scale=None if w.scale is None else w.scale.cpu().numpy())


def check_against_oracle(w: W.Workload, g_index, g_score, use_mask=True, rows=None, label="", tau=None, removed=None,
                         min_strict=None):
    """The acceptance rule at the dtype tolerance and at the tight one.  Returns the report at the dtype tolerance;
    its attribute `tight` is the report at the tight one.  min_strict: smallest fraction of the queries that the
    tight run must decide by exact index-set equality (for workloads without built-in exact ties)."""
    code = CODE[w.keys.dtype]
    full = oracle_scores(w, rows)
    if removed is not None:                 # removed entries are never candidates
        full = kb_oracle.without_removed(full, removed)
    tags = W.word_bits(w.tags) if (use_mask and w.qmask is not None) else None
    qm = W.word_bits(w.qmask) if (use_mask and w.qmask is not None) else None
    if rows is not None:
        g_index, g_score = g_index[rows], g_score[rows]
        qm = None if qm is None else qm[rows]
    tight = TIGHT_FP8_QUERIES if w.queries.dtype == torch.float8_e4m3fn else TIGHT
    rep, rep_tight = compare.check(g_index, g_score, full, w.k, TAU[code] if tau is None else tau, tags=tags, qmask=qm, label=label,
                                   tight_tau=tight)
    assert rep.max_score_err <= tight, f"{label}: passes the dtype tolerance but score error {rep.max_score_err:.2e} is suspicious"
    if min_strict is not None:
        assert rep_tight.strict >= min_strict * rep_tight.queries, (
            f"{label}: only {rep_tight.strict} of {rep_tight.queries} queries were decided by index-set equality at tau {tight:.0e}")
    rep.tight = rep_tight
    return rep


def run_and_check(w: W.Workload, use_mask=True, label="", tuning=None):
    kb = build_kb(w)
    for name, val in (tuning or {}).items():
        kb.set_tuning(name, val)
    gi, gs = gpu_query(kb, w, use_mask)
    if not tuning:
        # a small knowledge base is scored whole without sampling and candidate lists; the scan pipeline must give
        # the same bits (its counters are the ones reported)
        kb.set_tuning("small_path", 0)
        gi2, gs2 = gpu_query(kb, w, use_mask)
        assert np.array_equal(gi, gi2) and np.array_equal(gs.view(np.int32), gs2.view(np.int32)), f"{label}: the two pipelines disagree"
    rep = check_against_oracle(w, gi, gs, use_mask, label=label)
    counters = kb.counters()
    kb.close()
    return rep, counters, (gi, gs)
