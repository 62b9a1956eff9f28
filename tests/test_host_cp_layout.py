"""The C-ABI layout-conversion planner against its oracle (host only, no GPU)."""
import numpy as np
import pytest

from oracle import cp_layout_oracle as lo
from paper_2605_25451_amd import binding as bm
from paper_2605_25451_amd import synth
from tests.test_oracle_cp_layout import make_case


@pytest.mark.parametrize("enc_cp,llm_cp", [(1, 1), (1, 2), (2, 1), (2, 4), (3, 2), (4, 4), (8, 3)])
@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_plan_matches_oracle(enc_cp, llm_cp, seed):
    image_lens, image_rows, doc_lens = make_case(seed, n_docs=4)
    counts, src, dst = bm.cp_conversion_plan(enc_cp, llm_cp, image_lens, image_rows, synth.cu_from_lengths(doc_lens))
    rc, moves = lo.conversion_plan(image_lens, image_rows, doc_lens, enc_cp, llm_cp)
    assert counts.tolist() == rc
    o = 0
    for e in range(enc_cp):
        for l in range(llm_cp):
            n = rc[e][l]
            assert list(zip(src[o:o + n].tolist(), dst[o:o + n].tolist())) == moves[(e, l)]
            o += n
    assert o == sum(image_lens)


def test_plan_with_shuffled_rows_and_empty_images():
    # image tokens placed at arbitrary distinct rows, an image without tokens, a short document
    rng = np.random.default_rng(9)
    image_lens = [5, 0, 9, 1]
    doc_lens = [2, 30, 7]
    rows = rng.permutation(sum(doc_lens))[:sum(image_lens)].astype(np.int32)
    counts, src, dst = bm.cp_conversion_plan(3, 4, image_lens, rows, synth.cu_from_lengths(doc_lens))
    rc, moves = lo.conversion_plan(image_lens, rows, doc_lens, 3, 4)
    assert counts.tolist() == rc
    flat = [m for e in range(3) for l in range(4) for m in moves[(e, l)]]
    assert list(zip(src.tolist(), dst.tolist())) == flat


def test_plan_errors_and_unit_size():
    cu = synth.cu_from_lengths([4, 4])
    with pytest.raises(bm.BmError):
        bm.cp_conversion_plan(2, 2, [3], [0, 1, 1], cu)          # a row filled twice
    with pytest.raises(bm.BmError):
        bm.cp_conversion_plan(2, 2, [3], [0, 1, 8], cu)          # outside the pack
    with pytest.raises(bm.BmError):
        bm.cp_conversion_plan(0, 2, [3], [0, 1, 2], cu)
    assert bm.cp_encoder_unit_size(4, 2, 1) == 8
    assert bm.cp_encoder_unit_size(4, 2, 2) == lo.encoder_unit_size(4, 2, 2)
    with pytest.raises(bm.BmError):
        bm.cp_encoder_unit_size(3, 1, 2)
