"""GPU parity on reduced copies of the benchmark configurations 1-3 (the same shape rules, value
recipes and grids, leading dimensions shrunk so that the CPU oracle finishes in seconds):
ResNet-50-shaped weights with Adam state, BERT-base-shaped tensors whose word embedding moves on a
Zipf-drawn 5 % of its rows, and a GPT-2-medium-shaped five-step sequence with four deltas."""
import itertools
import os

import numpy as np
import pytest
import torch

from paper_2306_11800_amd import synth
from test_gpu_parity import check_delta, check_quantized, check_scores, dev, run_pipeline

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2306_11800_amd import api
    c = api.Context(torch.device("cuda:0"))
    yield c
    c.close()


def test_resnet50_shaped_with_adam_state(ctx):
    # 161 parameter tensors x (w, m, v), from 4-element biases to the 2048-wide last stage
    items = list(synth.resnet50_checkpoint(scale=1.0 / 32))
    items = items[:60] + items[-30:]
    prevs = [p for _, p, _ in items]
    curs = [c for _, _, c in items]
    assert min(p.size for p in prevs) < 100 and max(p.size for p in prevs) > 30_000
    run_pipeline(ctx, prevs, curs, synth.grid_small(), synth.EPS_DEFAULT, want_perm=False)


def test_bert_shaped_embedding_moves_on_few_rows(ctx):
    gen = synth.bert_base_checkpoint(scale=1.0 / 48)
    items = list(itertools.islice(gen, 0, 27))  # embeddings and the first encoder layer, with m and v
    names = [n for n, _, _ in items]
    assert "embeddings.word" in names and "embeddings.word.adam_m" in names
    prevs = [p for _, p, _ in items]
    curs = [c for _, _, c in items]
    w_prev, w_cur = prevs[names.index("embeddings.word")], curs[names.index("embeddings.word")]
    assert 0.9 < float(np.mean(w_prev == w_cur)) < 0.97  # 95 % of the rows do not move
    run_pipeline(ctx, prevs, curs, synth.grid_full(), synth.EPS_DEFAULT, want_perm=False)


def test_gpt2_shaped_five_steps_four_deltas(ctx):
    from oracle import ref
    gen = synth.gpt2_medium_steps(scale=1.0 / 160)
    items = list(itertools.islice(gen, 0, 9))  # wte, wpe and the first tensor of block 0, with m and v
    grid, eps = synth.grid_full(), synth.EPS_DEFAULT
    n_steps = len(items[0][1])
    assert n_steps == 5
    q_prev = r_prev = c_prev = None
    for t in range(n_steps):
        xs = [steps[t] for _, steps in items]
        ts = [dev(x) for x in xs]
        best, feas, scores = ctx.search(ts, grid, eps)
        chosen = [grid[check_scores(scores, len(grid), i, x, grid, eps, best[i], feas[i])]
                  for i, x in enumerate(xs)]
        qs = ctx.quantize(ts, chosen, reuse_search=True)
        refs = [check_quantized(q, x, c) for q, x, c in zip(qs, xs, chosen)]
        if q_prev is not None:
            ds = ctx.delta(q_prev, qs)
            ctx.sync()
            for i, d in enumerate(ds):
                check_delta(d, r_prev[i], c_prev[i][0], refs[i], chosen[i][0], False)
        q_prev, r_prev, c_prev = qs, refs, chosen


def test_resnet50_shaped_full_size(ctx):
    """Configuration 1 at its full size (483 tensors, 76.7 M values, the 24-configuration grid),
    searched, quantized and delta-encoded as one batch; the oracle runs one tensor per thread."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import ref
    items = list(synth.resnet50_checkpoint())
    prevs = [p for _, p, _ in items]
    curs = [c for _, _, c in items]
    assert len(items) == 483 and sum(p.size for p in prevs) > 76_000_000
    grid, eps = synth.grid_small(), synth.EPS_DEFAULT
    ref.lib()
    work = min(16, os.cpu_count() or 1)
    sides = []
    for xs in (prevs, curs):
        ts = [dev(x) for x in xs]
        best, feas, scores = ctx.search(ts, grid, eps)
        with ThreadPoolExecutor(work) as ex:
            rsearch = list(ex.map(lambda x: ref.search(x, grid, eps), xs))
        chosen = [grid[check_scores(scores, len(grid), i, x, grid, eps, best[i], feas[i], given=rsearch[i])]
                  for i, x in enumerate(xs)]
        qs = ctx.quantize(ts, chosen, reuse_search=True)
        with ThreadPoolExecutor(work) as ex:
            rq = list(ex.map(lambda xc: ref.quantize(xc[0], xc[1]), zip(xs, chosen)))
        refs = [check_quantized(q, x, c, given=r) for q, x, c, r in zip(qs, xs, chosen, rq)]
        sides.append((qs, refs, chosen))
        del ts
    (qp, rp, cp), (qc, rc, cc) = sides
    ds = ctx.delta(qp, qc)
    ctx.sync()
    with ThreadPoolExecutor(work) as ex:
        rd = list(ex.map(lambda k: ref.delta(rp[k]["sym"], cp[k][0], rc[k]["sym"], cc[k][0]), range(len(ds))))
    for i, d in enumerate(ds):
        check_delta(d, rp[i], cp[i][0], rc[i], cc[i][0], False, given=rd[i])
