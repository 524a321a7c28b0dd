"""Pins for oracle/maps.py: a case small enough to write out by hand, structural
invariants, and the error paths."""
from types import SimpleNamespace as NS

import numpy as np
import pytest

from oracle.maps import build_maps, check_attention_cover
from workload import gen


def R(kind, seq, start, n, adapter=-1):
    return NS(kind=kind, seq_id=seq, start_pos=start, n_new=n, adapter=adapter)


def test_hand_computed_case():
    # page size 4; seq 0: decode token at position 5 (pages 7, 2); seq 1: prefill chunk
    # of 3 tokens from position 2 (pages 0, 5); seq 2: finetune window of 2 tokens from
    # position 4 with adapter 0 (pages 3, 1)
    m = build_maps([R(0, 0, 5, 1), R(1, 1, 2, 3), R(2, 2, 4, 2, 0)],
                   {0: [7, 2], 1: [0, 5], 2: [3, 1]}, 4)
    assert m["T"] == 6 and m["n_req"] == 3 and m["n_ft"] == 2
    assert m["tok_req"].tolist() == [0, 1, 1, 1, 2, 2]
    assert m["tok_pos"].tolist() == [5, 2, 3, 4, 4, 5]
    assert m["req_tok_off"].tolist() == [0, 1, 4, 6]
    assert m["req_kv_len"].tolist() == [6, 5, 6]
    # slots: pos 5 -> page 2, off 1 -> 9 ; pos 2,3 -> page 0 -> 2,3 ; pos 4 -> page 5 -> 20 ;
    #        pos 4,5 -> page 1 -> 4,5
    assert m["slot"].tolist() == [9, 2, 3, 20, 4, 5]
    assert m["block_table"].tolist() == [[7, 2], [0, 5], [3, 1]]
    assert m["ft_tok"].tolist() == [4, 5]
    assert m["seg_off"].tolist() == [0, 4, 6]
    assert m["seg_adapter"].tolist() == [-1, 0]
    for k in ("tok_req", "tok_pos", "slot", "block_table", "ft_tok", "seg_off", "seg_adapter"):
        assert m[k].dtype == np.int32


def test_block_table_padding_and_unused_capacity():
    m = build_maps([R(0, 0, 0, 1), R(1, 1, 0, 9)], {0: [4, 9, 9], 1: [0, 1, 2, 3]}, 4)
    assert m["block_table"].tolist() == [[4, -1, -1], [0, 1, 2]]
    assert m["max_pages"] == 3


def test_segments_merge_equal_adapters():
    m = build_maps([R(2, 0, 0, 2, 1), R(2, 1, 0, 3, 1), R(0, 2, 3, 1, -1), R(2, 3, 0, 1, 0)],
                   {0: [0], 1: [1], 2: [2], 3: [3]}, 4)
    assert m["seg_off"].tolist() == [0, 5, 6, 7]
    assert m["seg_adapter"].tolist() == [1, -1, 0]


def test_named_batches_are_consistent():
    for b in (gen.batch_c1(0), gen.batch_c2(0)):
        m = build_maps(b.requests, b.seq_pages, b.page_size, b.num_pages)
        assert m["T"] == b.n_tokens and m["n_ft"] == b.n_ft_tokens
        assert len(set(m["slot"].tolist())) == m["T"]                       # injective
        assert np.all(np.diff(m["req_tok_off"]) == [r.n_new for r in b.requests])
        pos = m["tok_pos"]; ps = b.page_size
        bt = m["block_table"][m["tok_req"], pos // ps]
        assert np.array_equal(bt * ps + pos % ps, m["slot"])
    b = gen.batch_c2(0)
    assert b.n_tokens == 1024 and b.n_ft_tokens == 256 and len(b.requests) == 259


@pytest.mark.parametrize("reqs,pages,num_pages", [
    ([R(0, 0, 8, 1)], {0: [1, 2]}, 4),                       # kv_len 9 needs 3 pages
    ([R(0, 0, 0, 1)], {0: [4]}, 4),                          # page id out of range
    ([R(0, 0, 0, 1)], {0: [-1]}, 4),
    ([R(0, 0, 0, 1), R(0, 1, 0, 1)], {0: [1], 1: [1]}, 4),   # two sequences share a page
    ([R(1, 0, 0, 3), R(1, 0, 2, 2)], {0: [1, 2]}, 4),        # overlapping positions
    ([R(0, 0, 0, 0)], {0: [1]}, 4),
    ([R(3, 0, 0, 1)], {0: [1]}, 4),
    ([R(0, 5, 0, 1)], {0: [1]}, 4),
])
def test_invalid_descriptions_raise(reqs, pages, num_pages):
    with pytest.raises(ValueError):
        build_maps(reqs, pages, 4, num_pages)


def test_attention_cover_checker():
    m = build_maps([R(0, 0, 5, 1), R(1, 1, 2, 3)], {0: [0, 1], 1: [2, 3]}, 4)
    good = [(0, 1, 0, 4), (0, 1, 4, 6), (1, 4, 0, 5)]
    assert check_attention_cover(m, good)
    with pytest.raises(ValueError):
        check_attention_cover(m, good[:2])                 # request 1 missing
    with pytest.raises(ValueError):
        check_attention_cover(m, good + [(0, 1, 3, 5)])    # overlap
    with pytest.raises(ValueError):
        check_attention_cover(m, [(0, 2, 0, 6), (2, 4, 0, 5)])   # item spans two requests
