"""CPU oracle for the encoder -> LLM context-parallel layout conversion and the encoder unit size.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, never by the product path, and sharing no code
with it.

Sec. 3.3 "Context parallelism": encoder and LLM may use different context-parallel degrees; the
handoff then moves every modality embedding from the encoder ranks' layout to the LLM ranks'
layout with an all-to-all, and the encoder scheduling unit grows from pp_size to
pp_size * llm_cp / enc_cp microbatches.  The paper gives no layout; reading (same rule as for
attention): a sequence of length L is cut into C contiguous position ranges, chunk c holding
positions [c*L // C, (c+1)*L // C).  The encoder's sequences are the images (their patch tokens),
the LLM's are the documents; a rank's buffer holds its chunk of every sequence, sequence by
sequence.  An encoder token is identified by (image, patch position) and lands on the LLM row the
microbatch assigns to it.

Everything here is done the slow way: every token's source rank / row and destination rank / row
are found by enumerating the two layouts.
"""
from __future__ import annotations

import numpy as np


def chunk_layout(lens, C):
    """For sequences of the given lengths: owner[s][p] = (rank, local row) of position p of
    sequence s when every sequence is cut into C contiguous ranges and a rank stores its ranges
    sequence by sequence."""
    fill = [0] * C
    owner = []
    for L in lens:
        rows = [None] * L
        for c in range(C):
            for p in range(c * L // C, (c + 1) * L // C):
                rows[p] = (c, fill[c])
                fill[c] += 1
        owner.append(rows)
    return owner, fill


def conversion_plan(image_lens, image_rows, doc_lens, enc_cp, llm_cp):
    """image_rows[k]: row of the LLM pack (documents back to back) that encoder token k fills,
    tokens counted image by image.  Returns (counts [enc_cp][llm_cp], moves): moves[(e, l)] is the
    list of (source row on encoder rank e, destination row on LLM rank l), in source-row order."""
    enc_owner, _ = chunk_layout(image_lens, enc_cp)
    llm_owner, _ = chunk_layout(doc_lens, llm_cp)
    # LLM pack row -> (document, position)
    where = []
    for d, L in enumerate(doc_lens):
        where += [(d, p) for p in range(L)]
    moves = {(e, l): [] for e in range(enc_cp) for l in range(llm_cp)}
    k = 0
    for i, L in enumerate(image_lens):
        for p in range(L):
            e, src = enc_owner[i][p]
            d, q = where[int(image_rows[k])]
            l, dst = llm_owner[d][q]
            moves[(e, l)].append((src, dst))
            k += 1
    for key in moves:
        moves[key].sort()
    counts = [[len(moves[(e, l)]) for l in range(llm_cp)] for e in range(enc_cp)]
    return counts, moves


def encoder_unit_size(pp_size, llm_cp, enc_cp):
    """Microbatches per encoder unit: the LLM ranks of one context-parallel group consume the same
    encoder outputs in lockstep (Sec. 3.3; llm_cp 2, enc_cp 1, pp 4 gives 8)."""
    n = pp_size * llm_cp
    if n % enc_cp:
        raise ValueError("pp_size * llm_cp must be a multiple of enc_cp")
    return n // enc_cp
