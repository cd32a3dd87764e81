"""Host-side model of the dS scratch of the MFMA attention backward (csrc/attn_mfma.hip, csrc/attn_mfma_dq.hip).

The dK/dV kernel leaves dS in 4 KB blocks indexed [32-key block row][64-query step]; the dQ kernel reads them back
without any mask.  That is only right if (a) every block a dQ wavefront uses was written by the dK/dV kernel, (b) the
blocks it uses cover every (key, query) pair the attention mask admits, and (c) every address either kernel forms,
the never-used clamped loads of the dQ kernel included, lies inside the scratch.  The block arithmetic of the two
kernels is restated here and checked by brute force over segment layouts chosen around the tile sizes (32, 64, 128,
256).  The GPU parity tests check the values; this test checks the index argument at many more layouts than they run."""
import itertools

import numpy as np
import pytest

KV_TILE, Q_TILE = 128, 256          # rows per key tile (dK/dV workgroup) and per query tile (dQ workgroup)


def _cdiv(a, b):
    return -(-a // b)


def _segments(cu):
    kb0 = 0
    for s0, s1 in zip(cu[:-1], cu[1:]):
        yield s0, s1, kb0
        kb0 += _cdiv(s1 - s0, 32)


def written_blocks(cu, causal):
    """Blocks (row, step) the dK/dV kernel writes: wavefront w of a key tile owns keys r0 + 32 w .. + 31."""
    out = set()
    for s0, s1, kb0 in _segments(cu):
        for r0 in range(s0, s1, KV_TILE):
            r1 = min(r0 + KV_TILE, s1)
            q_begin = r0 if causal else s0
            nq_steps = _cdiv(s1 - q_begin, 64)
            for w in range(4):
                wj0 = r0 + 32 * w
                if wj0 >= r1:
                    continue                                   # no keys: every step skipped
                n_skip = min(nq_steps, (wj0 - q_begin) // 64) if causal else 0
                for t in range(n_skip, nq_steps):
                    q0 = q_begin + 64 * t
                    assert (q0 - s0) % 64 == 0 and (wj0 - s0) % 32 == 0
                    out.add((kb0 + (wj0 - s0) // 32, (q0 - s0) // 64))
    return out


def dq_wavefronts(cu, causal):
    """Per dQ wavefront: (segment, first query, step column, 32-row half, block rows used, block rows addressed)."""
    for s0, s1, kb0 in _segments(cu):
        for r0 in range(s0, s1, Q_TILE):
            r1 = min(r0 + Q_TILE, s1)
            kv_end = r1 if causal else s1
            nsteps = _cdiv(kv_end - s0, 128)
            nblk_all = _cdiv(kv_end - s0, 32)
            for w in range(8):
                wq0 = r0 + 32 * w
                has_rows = wq0 < r1
                nblk = 0 if not has_rows else (min(nblk_all, (wq0 - s0) // 32 + 1) if causal else nblk_all)
                used = [kb0 + kb for kb in range(nblk)]
                addressed = sorted({kb0 + min(kb, max(nblk - 1, 0)) for kb in range(4 * nsteps)})
                yield (s0, s1, r1), wq0, (wq0 - s0) // 64, ((wq0 - s0) // 32) & 1, used, addressed


LAYOUTS = [[0, n] for n in (1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 193, 255, 256, 257, 300, 511, 513, 777, 1100)]
LAYOUTS += [[0, a, a + b] for a, b in itertools.product((1, 5, 37, 64, 130, 257), (1, 33, 128, 259, 391))]
LAYOUTS += [[0, 1, 2, 3, 131], [0, 100, 200, 300, 600, 601], list(range(0, 785 * 8, 784))]


@pytest.mark.parametrize("causal", [True, False])
def test_dq_reads_only_written_blocks_and_covers_every_admitted_pair(causal):
    for cu in LAYOUTS:
        T, n_seg = cu[-1], len(cu) - 1
        ds_rows, ds_nqs = _cdiv(T, 32) + n_seg, _cdiv(T, 64) + 4          # attn_ds_rows / attn_ds_nqs with no slack in n_seg
        wr = written_blocks(cu, causal)
        assert all(0 <= r < ds_rows and 0 <= c < ds_nqs - 4 for r, c in wr), cu
        for (s0, s1, r1), wq0, col, half, used, addressed in dq_wavefronts(cu, causal):
            assert all(0 <= r < ds_rows for r in addressed) and 0 <= col < ds_nqs, (cu, wq0)
            for r in used:
                assert (r, col) in wr, (cu, causal, wq0, r, col)
            # every key the mask admits for a query of this wavefront lies in a used block row
            seg_kb0 = next(k for a, b, k in _segments(cu) if a == s0)
            for i in range(wq0, min(wq0 + 32, r1)):
                last_key = i if causal else s1 - 1
                assert seg_kb0 + (last_key - s0) // 32 in used, (cu, causal, i)
                assert seg_kb0 in used


def test_block_rows_of_different_segments_do_not_collide():
    rng = np.random.default_rng(5)
    for _ in range(200):
        lens = rng.integers(1, 400, size=rng.integers(1, 7))
        cu = [0] + list(np.cumsum(lens))
        rows = [set(range(kb0, kb0 + _cdiv(s1 - s0, 32))) for s0, s1, kb0 in _segments(cu)]
        assert sum(len(r) for r in rows) == len(set().union(*rows))
        assert max(max(r) for r in rows) < _cdiv(cu[-1], 32) + len(lens)
