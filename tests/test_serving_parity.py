"""The C++ scheduler and block manager against the Python oracle, operation by operation (CPU only):
identical chunks, identical block ids, copies, reuse counts and eviction choices."""
import numpy as np
import pytest

from oracle import serving as S
from paper_2412_18106_amd import binding as X


@pytest.mark.parametrize("seed", range(40))
def test_schedule_chunk_matches_the_oracle(seed):
    rng = np.random.default_rng(seed)
    t = int(rng.integers(1, 3000))
    r = int(rng.integers(0, t + 1))
    queue = []
    for i in range(int(rng.integers(0, 80))):
        kind = int(rng.integers(0, 3))
        tokens = int(rng.integers(1, 5000)) if kind == 0 else 1 if kind == 1 else int(rng.integers(1, 64))
        queue.append((1000 + i, kind, tokens, int(rng.integers(0, 40000))))
    assert X.xy_serve_schedule_chunk(t, r, queue) == S.schedule_chunk(t, r, queue)


def test_schedule_chunk_errors():
    for args in ((0, 0, []), (8, 9, []), (8, -1, []), (8, 2, [(1, 1, 2, 0)]), (8, 2, [(1, 0, 0, 0)]),
                 (8, 2, [(1, 5, 1, 0)]), (8, 2, [(1, 0, 4, -1)])):
        with pytest.raises(X.XyError) as e:
            X.xy_serve_schedule_chunk(*args)
        assert e.value.status == X.XY_ERR_ARG
    assert X.xy_serve_schedule_chunk(8, 2, []) == []


@pytest.mark.parametrize("seed", range(16))
def test_block_manager_matches_the_oracle_on_random_traffic(seed):
    rng = np.random.default_rng(500 + seed)
    b = int(rng.choice([2, 4, 16]))
    nblocks = int(rng.integers(16, 120))
    ref, lib = S.BlockManagerOracle(nblocks, b), X.KvManager(nblocks, b)
    library = [list(map(int, rng.integers(0, 4, size=int(rng.integers(3, 12 * b))))) for _ in range(5)]
    live = {}                                   # oracle seq id -> library seq id
    for _ in range(400):
        op = rng.random()
        if op < 0.3 or not live:
            base = library[int(rng.integers(0, len(library)))]
            toks = base[:int(rng.integers(1, len(base) + 1))] + list(map(int, rng.integers(0, 4, size=int(rng.integers(0, 2 * b)))))
            want = ref.open(toks)
            if want is None:
                with pytest.raises(X.XyError) as e:
                    lib.open(toks)
                assert e.value.status == X.XY_ERR_CAPACITY
            else:
                got = lib.open(toks)
                assert (got[1], got[2]) == (want[1], want[2])
                live[want[0]] = got[0]
                rest = toks[want[1]:]
                ok = ref.extend(want[0], rest)
                if ok:
                    lib.extend(got[0], rest)
                else:
                    with pytest.raises(X.XyError):
                        lib.extend(got[0], rest)
        elif op < 0.8:
            sid = list(live)[int(rng.integers(0, len(live)))]
            new = list(map(int, rng.integers(0, 4, size=int(rng.integers(0, 3 * b)))))
            ok = ref.extend(sid, new)
            if ok:
                lib.extend(live[sid], new)
            else:
                with pytest.raises(X.XyError) as e:
                    lib.extend(live[sid], new)
                assert e.value.status == X.XY_ERR_CAPACITY
        else:
            sid = list(live)[int(rng.integers(0, len(live)))]
            ref.close(sid)
            lib.close(live.pop(sid))
        for sid, lid in live.items():
            assert lib.block_row(lid) == ref.block_row(sid)
            assert lib.length(lid) == ref.length(sid)
        assert lib.stats() == ref.stats()
    lib.destroy()


def test_block_manager_errors():
    m = X.KvManager(4, 4)
    with pytest.raises(X.XyError):
        m.extend(99, [1])
    with pytest.raises(X.XyError):
        m.close(3)
    with pytest.raises(X.XyError):
        m.open([])
    with pytest.raises(X.XyError):
        X.KvManager(0, 4)
    seq, cached, copies = m.open([1, 2, 3])
    assert (cached, copies) == (0, [])
    with pytest.raises(X.XyError) as e:
        m.extend(seq, list(range(17)))          # needs 5 blocks of 4
    assert e.value.status == X.XY_ERR_CAPACITY
    assert m.block_row(seq) == [] and m.length(seq) == 0
    m.extend(seq, list(range(16)))
    assert m.block_row(seq) == [0, 1, 2, 3]
    m.destroy()
