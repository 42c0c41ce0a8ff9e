"""Pins of the oracle's adjacency mask M_adja (Alg. 1 step 14; Sec. 4.3; the reading stated at
``oracle.rsa_oracle.adjacency_mask``): closed forms where blocks and tiles coincide, and a
token-by-token brute force written independently of the oracle's tile-set formulation."""
import itertools

import numpy as np
import pytest

from oracle import rsa_oracle as ro
from paper_2511_19835_amd import synth


def _neighbours_along(n_tiles, i, radius):
    return min(i + radius, n_tiles - 1) - max(i - radius, 0) + 1


@pytest.mark.parametrize("grid,tile,radius", [((4, 16, 24), (2, 8, 8), 1), ((3, 8, 32), (1, 8, 8), 1),
                                              ((6, 16, 16), (2, 8, 8), 2), ((2, 8, 8), (2, 8, 8), 1)])
def test_blocks_equal_to_tiles_have_the_box_neighbourhood(grid, tile, radius):
    block = tile[0] * tile[1] * tile[2]
    coords = synth.tile_order_coords(grid, block, tile)
    part = ro.partition(coords.shape[0], 0, block)
    A = ro.adjacency_mask(coords, tile, part, radius)
    nt = [g // t for g, t in zip(grid, tile)]
    assert A.shape == (nt[0] * nt[1] * nt[2],) * 2
    assert np.array_equal(A, A.T) and A.diagonal().all()
    for n, (a, b, c) in enumerate(itertools.product(range(nt[0]), range(nt[1]), range(nt[2]))):
        expect = _neighbours_along(nt[0], a, radius) * _neighbours_along(nt[1], b, radius) * _neighbours_along(nt[2], c, radius)
        assert A[n].sum() == expect
        # the neighbours are exactly the tiles of the surrounding box, in raster numbering
        box = [(x * nt[1] + y) * nt[2] + z
               for x in range(max(a - radius, 0), min(a + radius, nt[0] - 1) + 1)
               for y in range(max(b - radius, 0), min(b + radius, nt[1] - 1) + 1)
               for z in range(max(c - radius, 0), min(c + radius, nt[2] - 1) + 1)]
        assert sorted(np.nonzero(A[n])[0].tolist()) == sorted(box)


@pytest.mark.parametrize("grid,tile,block,t_text", [((3, 5, 7), (2, 2, 4), 8, 0), ((2, 9, 10), (1, 4, 4), 16, 5),
                                                    ((5, 6, 6), (2, 8, 8), 32, 40), ((1, 12, 12), (1, 8, 8), 64, 0)])
def test_ragged_grid_matches_token_level_brute_force(grid, tile, block, t_text):
    coords = synth.tile_order_coords(grid, block, tile)
    tv = coords.shape[0]
    assert tv == grid[0] * grid[1] * grid[2]
    part = ro.partition(tv, t_text, block)
    A = ro.adjacency_mask(coords, tile, part, 1)
    N, M = part.n_video, part.n_blocks
    assert A.shape == (N, M)
    expect = np.zeros((N, M), dtype=bool)
    tiles = [tuple(int(c) // t for c, t in zip(coords[i], tile)) for i in range(tv)]
    for i in range(tv):
        for j in range(tv):
            if max(abs(a - b) for a, b in zip(tiles[i], tiles[j])) <= 1:
                expect[i // block, j // block] = True
    assert np.array_equal(A, expect)
    assert not A[:, N:].any()                      # text key blocks are never forced


def test_radius_zero_keeps_blocks_that_share_a_tile():
    grid, tile, block = (2, 8, 16), (2, 8, 8), 64       # every tile is cut into two blocks
    coords = synth.tile_order_coords(grid, block, tile)
    part = ro.partition(coords.shape[0], 0, block)
    A = ro.adjacency_mask(coords, tile, part, 0)
    assert np.array_equal(A, np.kron(np.eye(2, dtype=bool), np.ones((2, 2), dtype=bool)))


def test_forced_mask_only_adds_blocks_and_counts_toward_the_factor():
    rng = np.random.default_rng(3)
    grid, tile, block = (2, 8, 24), (1, 8, 8), 64
    coords = synth.tile_order_coords(grid, block, tile)
    part = ro.partition(coords.shape[0], 0, block)
    A_pool = rng.dirichlet(np.ones(part.n_blocks), size=part.n_video)
    adja = ro.adjacency_mask(coords, tile, part, 1)
    base = ro.select_blocks(A_pool, 0.5)
    full = ro.select_blocks(A_pool, 0.5, forced=adja)
    assert np.array_equal(full, base | adja)
    R0, R1 = ro.rectification_factor(A_pool, base), ro.rectification_factor(A_pool, full)
    np.testing.assert_allclose(R1 - R0, (A_pool * (adja & ~base)).sum(axis=1), rtol=0, atol=1e-15)


@pytest.mark.parametrize("grid,tile", [((3, 5, 7), (2, 2, 4)), ((4, 16, 16), (1, 8, 8)), ((5, 9, 17), (2, 8, 8))])
def test_tile_order_is_a_bijection_that_agrees_with_the_input_generator(grid, tile):
    order = ro.tile_order(grid, tile)
    tv = grid[0] * grid[1] * grid[2]
    assert sorted(order.tolist()) == list(range(tv))
    # the coordinates the synthetic inputs are drawn on are laid out in the same order
    coords = synth.tile_order_coords(grid, 64, tile)
    assert np.array_equal(order, (coords[:, 0] * grid[1] + coords[:, 1]) * grid[2] + coords[:, 2])
    # tokens of one tile are consecutive: along the order the tile index never decreases
    tile_id = ((coords[:, 0] // tile[0]) * 1000 + coords[:, 1] // tile[1]) * 1000 + coords[:, 2] // tile[2]
    assert (np.diff(tile_id) >= 0).all()


def test_reorder_round_trip_and_text_rows_stay():
    rng = np.random.default_rng(5)
    grid, tile = (3, 5, 7), (2, 2, 4)
    tv, tt = 105, 9
    X = rng.normal(size=(tv + tt, 4))
    Y = ro.reorder_tokens(X, grid, tile, 0)
    assert np.array_equal(Y[tv:], X[tv:]) and not np.array_equal(Y[:tv], X[:tv])
    assert np.array_equal(ro.reorder_tokens(Y, grid, tile, 1), X)
    # first tile of the order: t in {0,1}, h in {0,1}, w in {0..3}, raster inside the tile
    first = [(t * 5 + h) * 7 + w for t in range(2) for h in range(2) for w in range(4)]
    assert np.array_equal(Y[:16], X[first])
