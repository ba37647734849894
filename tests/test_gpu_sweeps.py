"""Parity of the paper-shaped sweep cases (prefix-cached prefill, chunked prefill, tree verification at
31 and 15 draft tokens, decode at a multi-head shape) against the fp64 oracle on sampled rows."""
import numpy as np
import pytest

from oracle import attention as A
from paper_2412_18106_amd import sweeps as S

pytestmark = pytest.mark.gpu
MAX_ABS = 2e-2


def pick(family, wanted):
    cases = {c[0]: c for c in S.FAMILIES[family]()}
    return [cases[n] for n in wanted]


CASES = (pick("prefix", ["prefix_prompt4096_cached0", "prefix_prompt8192_cached3072"])
         + pick("chunked", ["chunked_chunk4096_end16384"])
         + pick("verify", ["verify_b4_spec31_ctx4096", "verify_b4_spec31_ctx4096_one_unit_per_tree",
                           "verify_b8_spec15_ctx1024", "verify_b8_spec15_ctx1024_one_unit_per_tree"])
         + pick("decode", ["decode_h32_32_b8_ctx1024", "decode_h32_32_b32_ctx4096", "decode_h32_8_b128_ctx1024"])
         + pick("pages", ["pages_decode_h32_8_b128_ctx4096_page16", "pages_prefill_chunk2048_end16384_page32"]))


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_sweep_case_sampled_rows(case):
    import torch
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU")
    from paper_2412_18106_amd.runner import DeviceBatch
    name, hq, hkv, specs, overrides = case
    b = S.build_case(*case)
    db = DeviceBatch(b, **overrides)
    try:
        got = db.run_numpy()
    finally:
        db.close()
    assert not np.isnan(got).any()
    rng = np.random.default_rng(3)
    rows = [(0, 0, 0), (len(b.seqs) - 1, b.seqs[-1][0] - 1, hq - 1)]
    for _ in range(14):
        i = int(rng.integers(0, len(b.seqs)))
        rows.append((i, int(rng.integers(0, b.seqs[i][0])), int(rng.integers(0, hq))))
    ref = A.attention_oracle_rows(b.seqs, b.q, b.k_cache, b.v_cache, b.block_table, b.tree_masks, rows,
                                  num_q_heads=hq, num_kv_heads=hkv, block_size=b.block_size, scale=b.scale)
    starts = np.concatenate([[0], np.cumsum([s[0] for s in b.seqs])])
    for n, (i, r, h) in enumerate(rows):
        err = np.abs(got[starts[i] + r, h].astype(np.float64) - ref[n]).max()
        assert err <= MAX_ABS, f"{name}: row {(i, r, h)} max-abs {err:.3e}"
