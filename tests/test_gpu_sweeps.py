"""Parity of the paper-shaped sweep cases (prefix-cached prefill, chunked prefill, tree verification at
31 and 15 draft tokens, decode at a multi-head shape, small pages) against the fp64 oracle: every output
element of every sequence, max-abs and mean-abs per sequence."""
import pytest

from paper_2412_18106_amd import sweeps as S

import parity_util as PU

pytestmark = pytest.mark.gpu


def pick(family, wanted):
    cases = {c[0]: c for c in S.FAMILIES[family]()}
    return [cases[n] for n in wanted]


CASES = (pick("prefix", ["prefix_prompt4096_cached0", "prefix_prompt8192_cached3072"])
         + pick("chunked", ["chunked_chunk4096_end16384"])
         + pick("verify", ["verify_b4_spec31_ctx4096", "verify_b4_spec31_ctx4096_one_unit_per_tree",
                           "verify_b4_spec31_ctx16384",
                           "verify_b8_spec15_ctx1024", "verify_b8_spec15_ctx1024_one_unit_per_tree"])
         + pick("decode", ["decode_h32_32_b8_ctx1024", "decode_h32_32_b32_ctx4096", "decode_h32_8_b128_ctx1024"])
         + pick("pages", ["pages_decode_h32_8_b128_ctx4096_page16", "pages_prefill_chunk2048_end16384_page32"]))


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_sweep_case_every_row(case):
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
    every = list(range(len(b.seqs)))
    total, count, _ = PU.check_sequences(got, PU.oracle_sequences(b, every), b, every, name)
    assert count == got.size and total / count <= PU.MEAN_ABS
