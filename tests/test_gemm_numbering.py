"""Host-side enumeration of the block -> tile numbering of the grouped GEMMs (the code the kernels run, called
through the C ABI): every tile of a ragged map is computed exactly once, every K part of a split tile exactly
once, nothing is out of range, surplus blocks exit, and the fp32 partial sums of the split tiles stay inside
their workspace region.  Also the byte-offset bound of the weight-gradient GEMM's operand walk."""
import itertools

from paper_2504_03871_amd import binding as B

SPLIT_K, SPLIT_ROWS, NUM_XCD = 8, 64, 8


def test_row_tile_numbering_covers_every_tile_once():
    cases = itertools.product((0, 1, 5, 61, 64, 67), (0, 1, 3, 8), (1, 4, 16, 56))   # full tiles, partial tiles, column tiles
    for n_full, n_part, ntn in cases:
        for n_split in sorted({0, min(n_part, 1), n_part}):
            n_rt = n_full + n_part
            E = max(n_part, 1)
            grid = ntn * (n_rt + E) + E * ntn * (SPLIT_K - 1)        # the launch's worst-case block count
            seen, parts = {}, {}
            for vb in range(grid):
                ok, rt, _, nt, st, ks = B.moe_gemm_block_tile(0, vb, n_rt, n_full, n_split, 1, ntn)
                if not ok:
                    continue
                assert 0 <= rt < n_rt and 0 <= nt < ntn
                if st < 0:
                    assert rt < n_rt - n_split and (rt, nt) not in seen
                    seen[(rt, nt)] = vb
                else:
                    assert 0 <= st < n_split and rt == n_rt - n_split + st and 0 <= ks < SPLIT_K
                    assert (st, nt, ks) not in parts
                    parts[(st, nt, ks)] = vb
                    # fp32 partial sums: index of the last element this block may write, against the region
                    N = ntn * 256
                    last = ((st * SPLIT_K + ks) * SPLIT_ROWS + (SPLIT_ROWS - 1)) * N + (N - 1)
                    assert last * 4 < E * SPLIT_K * SPLIT_ROWS * N * 4
            assert len(seen) == (n_rt - n_split) * ntn and len(parts) == n_split * ntn * SPLIT_K
            # blocks of the full region that share an XCD (block % 8) get a contiguous run of tiles: walking an
            # XCD's blocks in dispatch order moves through row-tile groups of four, column by column
            per = (n_full * ntn) // NUM_XCD
            if per >= 8 and ntn >= 2 and n_full >= 4:
                x0 = [B.moe_gemm_block_tile(0, b, n_rt, n_full, n_split, 1, ntn) for b in range(0, 8 * NUM_XCD, NUM_XCD)]
                assert len({(t[1] // 4) for t in x0}) <= 2          # eight consecutive tiles of XCD 0: at most two groups


def test_weight_gradient_numbering_covers_every_tile_once_and_balances_xcds():
    for ntm, ntn, E in ((1, 1, 3), (4, 16, 2), (16, 56, 2), (56, 16, 1), (7, 5, 4), (3, 3, 5)):
        P = ntm * ntn
        P8 = (P + NUM_XCD - 1) // NUM_XCD * NUM_XCD
        seen = set()
        per_xcd = [[0] * NUM_XCD for _ in range(E)]
        for vb in range(P8 * E):
            ok, slot, mt, nt, _, _ = B.moe_gemm_block_tile(1, vb, ntm=ntm, ntn=ntn)
            if not ok:
                continue
            assert 0 <= slot < E and 0 <= mt < ntm and 0 <= nt < ntn and (slot, mt, nt) not in seen
            seen.add((slot, mt, nt))
            per_xcd[slot][vb % NUM_XCD] += 1
        assert len(seen) == P * E
        for e in range(E):      # an expert's tiles are spread evenly over the XCDs (skewed experts stay balanced)
            assert max(per_xcd[e]) - min(per_xcd[e]) <= 1
        if ntm >= 4 and ntn >= 8 and P8 // NUM_XCD >= 32:     # 32 tiles running together on XCD 0: a 4 x 8 patch
            t = [B.moe_gemm_block_tile(1, b, ntm=ntm, ntn=ntn) for b in range(0, 32 * NUM_XCD, NUM_XCD)]
            assert len({x[2] for x in t}) + len({x[3] for x in t}) <= 12 + 1


def test_rejects_bad_arguments():
    lib = B.lib()
    import ctypes
    out = (ctypes.c_int32 * 6)()
    assert lib.moe_gemm_block_tile(0, 0, 4, 5, 0, 1, 1, out) == -2        # more full tiles than tiles
    assert lib.moe_gemm_block_tile(0, 0, 4, 2, 3, 1, 1, out) == -2        # more split tiles than partial ones
    assert lib.moe_gemm_block_tile(2, 0, 4, 2, 0, 1, 1, out) == -3
    assert lib.moe_gemm_block_tile(0, 0, 4, 2, 0, 1, 1, None) == -1
