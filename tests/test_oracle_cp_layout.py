"""Pins for the context-parallel layout-conversion oracle (CPU only)."""
import numpy as np
import pytest

from oracle import cp_layout_oracle as lo
from paper_2605_25451_amd import synth


def make_case(seed, n_docs=3):
    """Documents of alternating image / text spans (config-3 recipe, small): returns image
    lengths, the LLM row of every image token, document lengths."""
    rng = np.random.default_rng(seed)
    image_lens, image_rows, doc_lens = [], [], []
    row = 0
    for _ in range(n_docs):
        L = 0
        for _ in range(int(rng.integers(1, 4))):
            li, lt = int(rng.integers(3, 20)), int(rng.integers(1, 9))
            image_lens.append(li)
            image_rows += list(range(row + L, row + L + li))
            L += li + lt
        doc_lens.append(L)
        row += L
    return image_lens, np.asarray(image_rows, dtype=np.int32), doc_lens


@pytest.mark.parametrize("enc_cp,llm_cp", [(1, 1), (1, 2), (2, 1), (2, 4), (3, 2), (4, 4)])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_plan_moves_every_token_to_its_llm_row(enc_cp, llm_cp, seed):
    image_lens, image_rows, doc_lens = make_case(seed)
    counts, moves = lo.conversion_plan(image_lens, image_rows, doc_lens, enc_cp, llm_cp)
    N = sum(image_lens)
    assert sum(map(sum, counts)) == N
    # label every encoder token by its global index, lay the labels out on the encoder ranks with the
    # library-independent partition of the input generator, move them, and compare with the direct
    # definition: LLM pack row image_rows[k] holds token k, then the pack is cut into LLM chunks
    enc_chunks = synth.context_chunks(synth.cu_from_lengths(image_lens), enc_cp)
    llm_chunks = synth.context_chunks(synth.cu_from_lengths(doc_lens), llm_cp)
    pack = np.full(sum(doc_lens), -1, dtype=np.int64)
    pack[image_rows] = np.arange(N)
    got = [np.full(len(rows), -1, dtype=np.int64) for rows, _ in llm_chunks]
    for (e, l), lst in moves.items():
        src_buf = enc_chunks[e][0]                       # global token index of every local row
        for src, dst in lst:
            assert got[l][dst] == -1                     # every destination row written once
            got[l][dst] = src_buf[src]
    for l, (rows, _) in enumerate(llm_chunks):
        assert np.array_equal(got[l], pack[rows])


def test_same_degree_and_aligned_sequences_stay_local():
    # one image per document and nothing else: both layouts cut the same sequences the same way
    image_lens = [8, 12, 5]
    rows = np.arange(sum(image_lens), dtype=np.int32)
    counts, moves = lo.conversion_plan(image_lens, rows, image_lens, 4, 4)
    for e in range(4):
        for l in range(4):
            assert (counts[e][l] == 0) == (e != l)
        assert all(s == d for s, d in moves[(e, e)])


def test_single_rank_sides():
    image_lens, image_rows, doc_lens = make_case(5)
    counts, moves = lo.conversion_plan(image_lens, image_rows, doc_lens, 1, 1)
    assert counts == [[sum(image_lens)]]
    assert [d for _, d in moves[(0, 0)]] == image_rows.tolist()      # plain scatter by image_rows


def test_encoder_unit_size():
    assert lo.encoder_unit_size(4, 2, 1) == 8          # the paper's example (Sec. 3.3, its CP figure)
    assert lo.encoder_unit_size(4, 1, 1) == 4
    assert lo.encoder_unit_size(4, 2, 2) == 4
    with pytest.raises(ValueError):
        lo.encoder_unit_size(3, 1, 2)


@pytest.mark.parametrize("C", [1, 2, 3, 4, 8])
def test_the_input_generators_partition_is_the_oracles_layout(C):
    """The seeded input module cuts packs into context-parallel chunks for the plumbing and the
    tests (synth.context_chunks); the oracle states the same rule on its own (chunk_layout).
    Both must describe one layout: rank c's k-th row of sequence s is the same pack row."""
    from paper_2605_25451_amd import synth
    rng = np.random.default_rng(100 + C)
    for lens in ([1], [7, 1, 2, 30], [C, C + 1, 2 * C - 1, 5 * C], rng.integers(1, 200, size=9).tolist()):
        cu = synth.cu_from_lengths(lens)
        chunks = synth.context_chunks(cu, C)
        owner, fill = lo.chunk_layout(lens, C)
        assert [len(rows) for rows, _ in chunks] == fill
        for c, (rows, cu_c) in enumerate(chunks):
            assert np.array_equal(np.diff(cu_c), [(c + 1) * L // C - c * L // C for L in lens])
        for s, L in enumerate(lens):
            for p in range(L):
                c, local = owner[s][p]
                assert chunks[c][0][local] == cu[s] + p, (s, p)
