"""Host logic of the context-parallel view: chunk bounds obey the rules of the range entry points
and partition every sequence; the pair count of a visit equals a brute-force count."""
import numpy as np

import cp_study


def test_chunk_ranges_partition_and_alignment():
    lengths = [1, 255, 256, 257, 1300, 5000, 40]
    for cp in (1, 2, 3, 4, 8):
        bounds = cp_study.chunk_ranges(lengths, cp, 256)
        for L, b in zip(lengths, bounds):
            assert len(b) == cp and b[0][0] == 0
            for c, (lo, hi) in enumerate(b):
                assert lo % 256 == 0 and hi >= lo
                assert hi % 256 == 0 or hi >= L
                if c + 1 < cp:
                    assert b[c + 1][0] == hi                 # contiguous
            assert b[-1][1] >= L                             # covers the sequence
            sizes = [max(0, min(hi, L) - lo) for lo, hi in b]
            assert sum(sizes) == L


def test_visit_pairs_against_brute_force():
    lengths = [700, 257, 1030, 40]
    for cp in (2, 3):
        bounds = cp_study.chunk_ranges(lengths, cp, 256)
        total = 0
        for r in range(cp):
            for c in range(cp):
                want = 0
                for L, b in zip(lengths, bounds):
                    i = np.arange(L)[:, None]; j = np.arange(L)[None, :]
                    m = (j <= i) & (i >= b[r][0]) & (i < b[r][1]) & (j >= b[c][0]) & (j < b[c][1])
                    want += int(m.sum())
                got = cp_study.visit_pairs(lengths, bounds, r, c)
                assert got == want, (cp, r, c)
                total += got
        assert total == sum(L * (L + 1) // 2 for L in lengths)


def test_zigzag_gives_every_rank_the_same_number_of_visible_blocks_and_all_pairs():
    for lengths, even in (([4096, 8192], True), ([4096, 700, 2049], False)):
      for cp in (2, 4):
        seen, counts = 0, []
        for r in range(cp):
            visits, n = cp_study.rank_visit_list(cp, r, True)
            assert n == 2 * cp and len(visits) == 2 * cp + 1
            bounds = cp_study.chunk_ranges(lengths, n, 256)
            counts.append(sum(cp_study.visit_pairs(lengths, bounds, a, b) for a, b in visits))
            seen += counts[-1]
        assert seen == sum(L * (L + 1) // 2 for L in lengths)          # the ranks together cover every pair once
        if even:                       # chunks of equal size: every rank holds exactly the same work
            assert max(counts) == min(counts)
        plain = []
        for r in range(cp):
            visits, n = cp_study.rank_visit_list(cp, r, False)
            bounds = cp_study.chunk_ranges(lengths, n, 256)
            plain.append(sum(cp_study.visit_pairs(lengths, bounds, a, b) for a, b in visits))
        assert sum(plain) == seen and max(plain) / min(plain) > 2.0    # contiguous chunks are not balanced
