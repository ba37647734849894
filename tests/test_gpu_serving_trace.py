"""A small synthetic serving trace end to end on the GPU: scheduler -> block manager -> plan -> copy-on-write
copies -> fused-QKV run.  The test keeps its own host mirror of the K/V cache (copies and appends applied
through the oracles) and checks, at every step, the device cache bit for bit and the attention output of
the step against the fp64 oracle."""
import numpy as np
import pytest

from oracle import attention as A
from oracle import kv_append as KA
from paper_2412_18106_amd import workloads as W

pytestmark = pytest.mark.gpu
MAX_ABS, MEAN_ABS = 2e-2, 2e-3


@pytest.mark.parametrize("block_size,num_blocks,speculative", [(16, 70, 0.0), (128, 40, 0.0), (16, 130, 0.6), (128, 48, 0.6)])
def test_trace_matches_the_oracles_step_by_step(block_size, num_blocks, speculative):
    import torch
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU")
    from paper_2412_18106_amd import serving as T
    hq, hkv, d = 8, 2, 128
    reqs = T.synthetic_requests(20, seed=3, prefix_lens=(150, 90), suffix=(10, 80),
                                outputs=(3, 10) if not speculative else (8, 40), vocab=50, arrivals_per_step=3,
                                speculative_fraction=speculative)
    pool = 0 if not speculative else (40 if block_size == 16 else 8)
    k_mirror = np.zeros((num_blocks, hkv, block_size, d), np.uint16)
    v_mirror = np.zeros_like(k_mirror)
    host_fused = {}
    seen = {"steps": 0, "rows": 0, "verify": 0, "trees": 0}

    def fused_fn(step, tokens):
        bits = W.noise_bf16([991, step], (tokens, hq + 2 * hkv, d))
        host_fused[step] = bits
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    def on_step(info):
        nonlocal k_mirror, v_mirror
        bits = host_fused.pop(info["step"])
        for src, dst, rows in info["copies"]:                        # copy-on-write, then this step's rows
            k_mirror[dst, :, :rows] = k_mirror[src, :, :rows]
            v_mirror[dst, :, :rows] = v_mirror[src, :, :rows]
        q, k_new, v_new = KA.split_fused_qkv(bits, hq, hkv)
        k_mirror, v_mirror = KA.append_kv_oracle(info["seqs"], k_new, v_new, k_mirror, v_mirror,
                                                 info["block_table"], block_size)
        k_dev = info["k_cache"].view(torch.int16).cpu().numpy().view(np.uint16)
        v_dev = info["v_cache"].view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(k_dev, k_mirror) and np.array_equal(v_dev, v_mirror), f"cache differs at step {info['step']}"
        ref = A.attention_oracle(info["seqs"], np.ascontiguousarray(q), k_mirror, v_mirror, info["block_table"],
                                 info["tree_masks"], num_q_heads=hq, num_kv_heads=hkv, block_size=block_size,
                                 scale=1.0 / np.sqrt(d))
        got = info["out"].float().cpu().numpy().astype(np.float64)
        err = np.abs(got - ref)
        assert not np.isnan(got).any() and err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, \
            f"step {info['step']}: max {err.max():.3e} mean {err.mean():.3e}"
        seen["steps"] += 1
        seen["rows"] += ref.shape[0]
        seen["verify"] += sum(1 for sq in info["seqs"] if sq[2] == W.VERIFY)
        seen["trees"] += sum(1 for sq in info["seqs"] if sq[3] == W.MASK_TREE)

    st = T.run_trace(reqs, num_q_heads=hq, num_kv_heads=hkv, num_blocks=num_blocks, block_size=block_size,
                     token_budget=128 if not speculative else 160, reserved_decode_slots=16 if not speculative else 64,
                     fused_fn=fused_fn, on_step=on_step, draft_pool_blocks=pool)
    assert st["finished"] == len(reqs) and st["open"] == 0
    assert seen["steps"] == st["steps"] and seen["rows"] == st["tokens"]
    assert st["tokens"] == st["prefill_tokens"] + st["decode_tokens"] + st["verify_tokens"]
    if speculative:
        # verify segments ran, chains and trees, some accepted rows had to be moved out of the draft pool, and every
        # accepted token is in the books
        assert seen["verify"] == st["verify_segments"] > 10 and 0 < seen["trees"] < seen["verify"]
        assert st["commit_copies"] > 0 and st["accepted_tokens"] >= st["verify_segments"] - st["lost_verify_segments"]
    else:
        assert st["verify_segments"] == 0
    assert st["prefill_tokens"] == st["prompt_tokens"] - st["reused_tokens"]
    assert st["reused_tokens"] > 0                     # shared prefixes were found in the cache
    if block_size == 16:
        assert st["cow_copies"] > 0                    # some prefix ended inside a block
        assert st["evictions"] > 0                     # the cache limit was reached
