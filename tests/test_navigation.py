"""Search-space navigation (Sec. 5: guided exhaustive search, Alg. 4; delta-neighbourhood search) of
the library's host code against brute force over the whole cube, on synthetic score tables.  With
quality and cost monotone along every axis the guided search must return the cheapest feasible cell
after reading only part of the cube; the neighbourhood search must return the cheapest feasible cell
of its neighbourhood."""
import itertools

import numpy as np
import pytest

from paper_2306_11800_amd import api, synth


def table(dims, rng, monotone=True):
    """Scores of a cube: sse falls and cost rises with every step along any axis (sums of positive
    increments), or unrelated numbers."""
    a, b, c = dims
    if monotone:
        q = (np.cumsum(rng.random(a) + 0.05)[:, None, None] + np.cumsum(rng.random(b) + 0.05)[None, :, None]
             + np.cumsum(rng.random(c) + 0.05)[None, None, :])
        cost = (np.cumsum(rng.integers(1, 50, a))[:, None, None] * 1000 + np.cumsum(rng.integers(1, 50, b))[None, :, None] * 37
                + np.cumsum(rng.integers(1, 50, c))[None, None, :])
        sse = q.max() + 0.1 - q
    else:
        sse = rng.random(dims) * 3
        cost = rng.integers(1, 10_000, dims)
    n = a * b * c
    perm = rng.permutation(n)                     # the grid lists the configurations in any order
    scores = (api.CScore * n)()
    cells = [0] * n
    for flat, (i, j, k) in enumerate(itertools.product(range(a), range(b), range(c))):
        g = int(perm[flat])
        cells[flat] = g
        scores[g].sse, scores[g].sumsq, scores[g].cost_bits = float(sse[i, j, k]), 1.0, int(cost[i, j, k])
    return scores, cells, sse, cost


def brute(sse, cost, eps, cells, dims, only=None):
    best = None
    for flat, ijk in enumerate(itertools.product(*(range(d) for d in dims))):
        if only is not None and ijk not in only:
            continue
        if sse[ijk] <= eps:
            key = (int(cost[ijk]), cells[flat])
            if best is None or key < best[0]:
                best = (key, ijk)
    return best


@pytest.mark.parametrize("dims", [(6, 6, 3), (1, 1, 1), (7, 1, 2), (1, 9, 1), (4, 5, 6), (2, 2, 2)])
def test_guided_search_finds_the_cheapest_feasible_cell_of_a_monotone_cube(dims):
    rng = np.random.default_rng(sum(dims))
    fewer = 0
    for trial in range(40):
        scores, cells, sse, cost = table(dims, rng)
        eps = float(rng.choice(sse.ravel())) if trial % 5 else float(sse.min()) - 1.0   # sometimes nothing is feasible
        cell, feas, trials, vis = api.guided_search(scores, cells, dims, eps)
        want = brute(sse, cost, eps, cells, dims)
        assert feas == (want is not None)
        if want is None:
            assert cell == tuple(d - 1 for d in dims)
        else:
            assert cost[cell] == want[0][0] and sse[cell] <= eps
            assert cell == want[1]          # (costs of a cube are distinct here up to the index tie-break)
        assert trials == sum(vis) <= np.prod(dims)
        fewer += trials < np.prod(dims)
    if np.prod(dims) >= 36:
        assert fewer >= 30                  # the point of the method: most cubes are not read whole


def test_guided_search_on_the_cube_of_the_paper_reads_a_fraction():
    grid = synth.grid_paper()
    cells, dims, axes = api.cube_of(grid)
    assert dims == (6, 6, 3) and axes[0] == [4, 6, 8, 12, 16, 32] and axes[1][0] == 500000 and axes[2][0] == 500
    assert sorted(cells) == list(range(108))
    rng = np.random.default_rng(7)
    reads = []
    for _ in range(50):
        scores, cells2, sse, cost = table(dims, rng)
        eps = float(np.quantile(sse, rng.random()))
        cell, feas, trials, _ = api.guided_search(scores, cells2, dims, eps)
        assert feas and cost[cell] == brute(sse, cost, eps, cells2, dims)[0][0]
        reads.append(trials)
    assert np.mean(reads) < 0.6 * 108


def test_guided_search_on_any_table_returns_a_feasible_cell_it_has_read():
    rng = np.random.default_rng(11)
    for _ in range(30):
        dims = tuple(int(x) for x in rng.integers(1, 7, 3))
        scores, cells, sse, cost = table(dims, rng, monotone=False)
        cell, feas, trials, vis = api.guided_search(scores, cells, dims, 1.5)
        flat = (cell[0] * dims[1] + cell[1]) * dims[2] + cell[2]
        if feas:
            assert sse[cell] <= 1.5 and vis[flat] == 1
        assert 1 <= trials <= np.prod(dims)


def neighbourhood(prev, e, dims):
    out = set()
    for ijk in itertools.product(*(range(d) for d in dims)):
        dist = sum(abs(x - y) for x, y in zip(ijk, prev))
        more_aggressive = all(x <= y for x, y in zip(ijk, prev)) and ijk != prev
        if dist <= e and not more_aggressive:
            out.add(ijk)
    return out


def test_neighbourhood_search_is_brute_force_over_its_cells():
    rng = np.random.default_rng(13)
    dims = (6, 6, 3)
    for trial in range(60):
        scores, cells, sse, cost = table(dims, rng, monotone=trial % 3 != 0)
        prev = tuple(int(rng.integers(0, d)) for d in dims)
        e = int(rng.integers(0, 4))
        eps = float(np.quantile(sse, rng.random()))
        cell, feas, trials = api.neighbourhood_search(scores, cells, dims, prev, e, eps)
        nb = neighbourhood(prev, e, dims)
        want = brute(sse, cost, eps, cells, dims, only=nb)
        assert feas == (want is not None)
        if want is None:
            assert cell == prev and trials == len(nb)
        else:
            assert cell == want[1]
            # read in ascending order of cost, stopping at the first feasible one
            order = sorted(nb, key=lambda ijk: (int(cost[ijk]), cells[(ijk[0] * dims[1] + ijk[1]) * dims[2] + ijk[2]]))
            assert trials == order.index(cell) + 1
    # e = 0: the previous configuration alone
    scores, cells, sse, cost = table(dims, rng)
    cell, feas, trials = api.neighbourhood_search(scores, cells, dims, (2, 3, 1), 0, float(sse.max()))
    assert (cell, feas, trials) == ((2, 3, 1), True, 1)


def test_navigation_argument_errors():
    scores, cells, sse, cost = table((2, 2, 2), np.random.default_rng(1))
    with pytest.raises(api.InshrError):
        api.guided_search(scores, cells, (0, 4, 2), 1.0) if False else api.neighbourhood_search(scores, cells, (2, 2, 2), (2, 0, 0), 1, 1.0)
    with pytest.raises(ValueError):
        api.guided_search(scores, cells, (2, 2, 3), 1.0)
