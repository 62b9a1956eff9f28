"""The layout-conversion plan applied on device memory with the C-ABI row moves (needs a GPU):
encoder-rank buffers -> per-pair send buffers -> LLM-rank buffers, bit-exact against the
definition (scatter into the full pack, then cut the pack into the LLM ranks' chunks)."""
import numpy as np
import pytest

from paper_2605_25451_amd import synth
from tests.test_oracle_cp_layout import make_case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [synth.DTYPE_BF16, synth.DTYPE_FP32], ids=["bf16", "fp32"])
@pytest.mark.parametrize("enc_cp,llm_cp", [(1, 2), (2, 4), (3, 2)])
def test_conversion_on_device(enc_cp, llm_cp, dtype):
    import torch
    from paper_2605_25451_amd import binding as bm
    from paper_2605_25451_amd.runner import to_device
    width = 64
    image_lens, image_rows, doc_lens = make_case(11, n_docs=5)
    N, T = sum(image_lens), sum(doc_lens)
    rng = np.random.default_rng(12)
    feat = synth.to_storage(rng.standard_normal((N, width), dtype=np.float32), dtype)     # encoder outputs, token order
    base = synth.to_storage(rng.standard_normal((T, width), dtype=np.float32), dtype)     # LLM rows before the handoff
    enc_chunks = synth.context_chunks(synth.cu_from_lengths(image_lens), enc_cp)
    llm_chunks = synth.context_chunks(synth.cu_from_lengths(doc_lens), llm_cp)
    counts, src, dst = bm.cp_conversion_plan(enc_cp, llm_cp, image_lens, image_rows, synth.cu_from_lengths(doc_lens))
    enc_buf = [to_device(feat[rows], dtype) for rows, _ in enc_chunks]
    llm_buf = [to_device(base[rows], dtype) for rows, _ in llm_chunks]
    o = 0
    for e in range(enc_cp):
        for l in range(llm_cp):
            n = int(counts[e, l])
            if n:
                s_dev = torch.from_numpy(src[o:o + n].copy()).cuda()
                d_dev = torch.from_numpy(dst[o:o + n].copy()).cuda()
                send = torch.empty((n, width), dtype=enc_buf[e].dtype, device="cuda")
                bm.row_gather(dtype, enc_buf[e], s_dev, send, n, width)        # what rank e sends to rank l
                bm.row_scatter(dtype, send, d_dev, llm_buf[l], n, width)      # where rank l puts it
            o += n
    torch.cuda.synchronize()
    want = base.copy()
    want[image_rows] = feat
    for l, (rows, _) in enumerate(llm_chunks):
        got = llm_buf[l].float().cpu().numpy()
        assert np.array_equal(got, want[rows].astype(np.float32))
