"""Host logic of the GEMM planner and of the variant menu (no GPU needed: these entry points only
compute).  What is checked is consistency -- every plan names a menu entry, workspace sizes follow
from the plan -- and the regime boundaries the design relies on, not the fitted constants."""
import random

import pytest


@pytest.fixture(scope="module")
def lg():
    import paper_2202_03293_amd as pkg
    pkg.lib()
    return pkg


def cdiv(a, b):
    return (a + b - 1) // b


def test_variant_menu_is_consistent(lg):
    n = lg.lg_gemm_variants()
    infos = [lg.lg_gemm_variant_info(v) for v in range(n)]
    assert len(set(infos)) == n
    for bm, bn, bk, parts, loop in infos:
        assert bm in (16, 32, 64, 128) and bn % 16 == 0 and bk in (16, 32) and parts in (1, 2, 4) and loop in (0, 1)
        assert parts == 1 or bm == 16                 # only the register-direct kernel cuts k inside a workgroup
        assert not loop or (bm, bn, bk, parts, 0) in infos   # a tile-loop variant is one of the tiles, looped
    for bad in (-1, n, n + 7):
        with pytest.raises(lg.LgError):
            lg.lg_gemm_variant_info(bad)


def test_plans_name_menu_entries_and_size_their_workspace(lg):
    infos = [lg.lg_gemm_variant_info(v) for v in range(lg.lg_gemm_variants())]
    blocks = {i[:2] for i in infos}
    loop_blocks = {i[:2] for i in infos if i[4]}
    rng = random.Random(5)
    shapes = [(rng.choice([1, 7, 64, 200, 1000, 4096, 30000]), rng.choice([1, 5, 32, 64, 256, 1024, 5000]),
               rng.choice([1, 3, 27, 64, 576, 2304, 8192, 50000])) for _ in range(300)]
    for M, N, K in shapes:
        bm, bn, splits = lg.lg_matmul_plan(M, N, K)
        assert (bm, bn) in blocks, (M, N, K)
        assert 1 <= splits <= max(1, cdiv(K, 128))
        # the workspace a caller is told to bring covers the plan of every operand layout
        need = lg.lg_matmul_workspace_bytes(M, N, K)
        plans = [(bm, bn, splits), lg.lg_matmul_t_plan(M, N, K, trans_a=True), lg.lg_matmul_t_plan(M, N, K, trans_b=True)]
        assert plans[1] == plans[0], (M, N, K)
        # (A B^T has no tile loop, which short contractions with a large output take in the other two layouts)
        assert plans[2][:2] in blocks
        assert need == max(sp * M * N * 4 if sp > 1 else 0 for _, _, sp in plans), (M, N, K)
        if bm == 16:
            assert splits == 1
    assert lg.lg_matmul_workspace_bytes(0, 4, 4) == 0


def test_regimes(lg):
    # chip-filling problems: LDS tiles, no split; a handful of output tiles: the register-direct kernel
    for shape in [(8192, 8192, 8192), (4096, 4096, 4096), (16384, 512, 2048)]:
        assert lg.lg_matmul_plan(*shape) == (128, 128, 1)
    for shape in [(64, 64, 64), (256, 256, 256), (196, 64, 288), (17, 33, 5)]:
        assert lg.lg_matmul_plan(*shape)[0] == 16
    # a short contraction with a large output: one of the tiles that have a tile loop; not so from K = 512 on
    loop_blocks = {i[:2] for i in (lg.lg_gemm_variant_info(v) for v in range(lg.lg_gemm_variants())) if i[4]}
    for shape in [(4096, 4096, 64), (8192, 8192, 128), (16384, 1024, 64)]:
        assert lg.lg_matmul_plan(*shape)[:2] in loop_blocks and lg.lg_matmul_plan_tile_loop(*shape)
    # ... nor with fewer than 256 rows, or with dense output rows that do not start on 128-byte boundaries
    for shape in [(4096, 4096, 512), (128, 100000, 64), (4096, 4100, 64), (4096, 4096, 66)]:
        assert not lg.lg_matmul_plan_tile_loop(*shape)
    # few tiles and a deep contraction: split along k
    assert lg.lg_matmul_plan(784, 512, 4608)[2] > 1
    # a few dozen rows against a large B stored N x K: tiles with k-slabs, where AB takes the direct blocks
    assert lg.lg_matmul_plan(64, 4096, 4096)[0] == 16
    bm, _, sp = lg.lg_matmul_t_plan(64, 4096, 4096, trans_b=True)
    assert bm > 16 and sp > 1
    assert lg.lg_matmul_workspace_bytes(64, 4096, 4096) == sp * 64 * 4096 * 4
    with pytest.raises(lg.LgError):
        lg.lg_matmul_t_plan(64, 64, 64, trans_a=True, trans_b=True)


def test_variant_workspace_follows_the_slab_rule(lg):
    n = lg.lg_gemm_variants()
    for v in range(n):
        info = lg.lg_gemm_variant_info(v)
        direct, loop = info[0] == 16, info[4] == 1
        for M, N, K, ks in [(100, 50, 1000, 4), (64, 64, 64, 2), (10, 10, 130, 3), (300, 200, 4096, 8)]:
            got = lg.lg_gemm_variant_workspace_bytes(M, N, K, v, ks)
            if direct or loop:                         # neither takes a k-split: nothing to bring
                assert got == 0
                continue
            per = cdiv(cdiv(K, 64), ks) * 64           # slabs are whole multiples of 64 k
            slabs = cdiv(K, per)
            assert got == (slabs * M * N * 4 if slabs > 1 else 0), (v, M, N, K, ks)
