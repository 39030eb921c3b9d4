"""The C ABI without a GPU: the library loads, exports every symbol the header declares,
and its host-side logic (configuration checks, sizes, closed-form exchange counts, ring
bookkeeping, error codes) behaves as documented.  No kernel is launched here."""
import os
import re
import subprocess
import sys

import numpy as np
import pytest

import oracle
import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    import paper_2512_19342_amd as pkg
    if not os.path.exists(pkg.lib_path()):          # build only when nothing is built
        from paper_2512_19342_amd import build
        build.build()
    return pkg


def test_every_declared_symbol_is_exported(B):
    header = open(os.path.join(ROOT, "include", "bls.h")).read()
    declared = set(re.findall(r"^(?:int|const char \*)\s*\*?(bls_\w+)\s*\(", header, re.M))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    lib = B.lib()
    for name in declared:
        assert getattr(lib, name) is not None
    out = subprocess.check_output(["nm", "-D", "--defined-only", B.lib_path()], text=True)
    exported = set(re.findall(r" T (bls_\w+)", out))
    assert exported == declared, exported ^ declared     # nothing else leaks out of the C ABI


def test_configuration_is_validated(B):
    ok = dict(P=2, T=3, D=8, k=1, B=4, rows=[5, 6, 7], table_owner=[0, 1, 0])
    B.Context(**ok).bls_destroy()
    bad = [dict(P=0), dict(P=65), dict(T=0, rows=[], table_owner=[]), dict(D=0), dict(k=-1), dict(B=1),
           dict(B=2 ** 31), dict(rows=[5, 0, 7]), dict(table_owner=[0, 2, 0]), dict(table_dtype=4), dict(part_kind=3)]
    for change in bad:
        with pytest.raises(B.BlsError):
            B.Context(**{**ok, **change})
    with pytest.raises(B.BlsError):                       # one grid row per (owner, table): F*T <= 65535
        B.Context(P=64, T=1024, D=4, k=1, B=64, rows=[9] * 1024, table_owner=[0] * 1024, part_kind=B.BLS_ROW_WISE)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_sizes_and_exchange_counts_match_oracle(B, cfg):
    w = synth.workload(cfg, "small" if cfg >= 3 else "full")
    c = B.Context(w.P, w.T, w.D, w.k, w.B, w.rows, w.table_owner,
                  w.dtype_code, w.part_kind)
    sz = c.bls_sizes(12345)
    n_float = w.F * w.T * w.B * w.D
    assert sz["pooled_bytes"] == sz["send_bytes"] == sz["slot_bytes"] == 4 * n_float
    assert sz["plan_ws_bytes"] >= 8 * (2 * w.P * w.P + w.F * w.T * w.P)      # bucket starts + a count per owner and run
    ref = oracle.pooled_counts(oracle.Case(w.P, w.T, w.D, w.B, w.part_kind, w.rows, w.table_owner))
    got = c.bls_pooled_counts()
    for k in ("pcount", "psdispl", "prcount", "prdispl"):
        assert got[k] == ref[k].tolist(), k
    assert sum(got["pcount"]) == n_float
    assert c.bls_ring_state() == (0, 0, max(w.k, 1))


def test_ring_bookkeeping_without_gpu(B):
    """Figure of the section on the bound: k = 3, three iterations may be started, the fourth must wait."""
    c = B.Context(3, 3, 4, 3, 6, [5, 5, 5], [0, 1, 2])
    with pytest.raises(B.BlsError) as e:
        c.bls_unpack(0, None, 0)
    assert e.value.code == B.BLS_ERING_EMPTY
    assert [c.bls_ring_advance(0) for _ in range(3)] == [(0, 0), (1, 1), (2, 2)]
    with pytest.raises(B.BlsError) as e:
        c.bls_ring_advance(0)
    assert e.value.code == B.BLS_ERING_FULL and "in flight" in c.bls_last_error()
    with pytest.raises(B.BlsError) as e:
        c.bls_unpack(1, None, 0)                          # not the oldest
    assert e.value.code == B.BLS_EORDER
    with pytest.raises(B.BlsError) as e:
        c.bls_unpack(0, None, 0)                          # oldest, but NULL output: rejected before any GPU call
    assert e.value.code == B.BLS_EINVAL
    assert c.bls_ring_state() == (3, 0, 3)
    for k in (0, 1):
        c1 = B.Context(2, 2, 4, k, 4, [5, 5], [0, 1])
        assert c1.bls_ring_state()[2] == 1                # k = 0 and k = 1: one slot
        assert c1.bls_ring_advance(0) == (0, 0)
        with pytest.raises(B.BlsError):
            c1.bls_ring_advance(0)


def test_partition_rule_hot_rows_and_tuning_without_gpu(B):
    """Host-side calls that touch no GPU: the row-wise partition rule as the library states it, the checks on
    hot-row lists and on the pool's tuning knobs, the size of the descriptor buffer, and the refusal of the
    plan without a workspace when the problem is too large for its static array."""
    c = B.Context(P=3, T=2, D=8, k=1, B=6, rows=[10, 4], table_owner=[0, 0], part_kind=B.BLS_ROW_WISE)
    # blocks of ceil(rows / P) rows; trailing shards short or empty
    assert [c.bls_shard_range(0, d) for d in range(3)] == [(0, 4), (4, 4), (8, 2)]
    assert [c.bls_shard_range(1, d) for d in range(3)] == [(0, 2), (2, 2), (4, 0)]
    for t, rows in ((0, 10), (1, 4)):                      # the blocks tile the table exactly
        spans = [c.bls_shard_range(t, d) for d in range(3)]
        assert sum(n for _, n in spans) == rows and all(spans[d][0] == min(d * -(-rows // 3), rows) for d in range(3))
    tw = B.Context(P=2, T=2, D=8, k=1, B=4, rows=[5, 6], table_owner=[1, 0])
    assert tw.bls_shard_range(0, 1) == (0, 5) and tw.bls_shard_range(0, 0) == (0, 0)
    with pytest.raises(B.BlsError):
        c.bls_shard_range(2, 0)
    base = c.bls_desc_bytes()
    assert 0 < base < 4096
    c.bls_set_hot_rows(0, 1, [3, 1, 3, 0])                 # a repeat is dropped
    assert c.bls_desc_bytes() >= base and c.bls_desc_bytes() <= base + 16
    with pytest.raises(B.BlsError) as e:
        c.bls_set_hot_rows(0, 2, [2])                      # shard (0, 2) has rows 0 and 1 only
    assert e.value.code == B.BLS_EINVAL
    with pytest.raises(B.BlsError):
        c.bls_set_hot_rows(1, 2, [0])                      # an empty shard
    with pytest.raises(B.BlsError):
        tw.bls_set_hot_rows(0, 0, [0])                     # not the table's owner
    c.bls_set_hot_rows(0, 1, [])                           # cleared
    assert c.bls_desc_bytes() == base
    c.bls_set_pool_tuning(lane_bytes=8, segments_per_group=3, xcd_map=0, wide_positions=1)
    for bad in (dict(lane_bytes=5), dict(segments_per_group=64), dict(xcd_map=2), dict(wide_positions=-2)):
        with pytest.raises(B.BlsError) as e:
            c.bls_set_pool_tuning(**bad)
        assert e.value.code == B.BLS_EINVAL
    for ok in (-1, 0, 1):
        c.bls_set_plan_tuning(ok)
    for bad in (-2, 2):
        with pytest.raises(B.BlsError) as e:
            c.bls_set_plan_tuning(bad)
        assert e.value.code == B.BLS_EINVAL
    big = B.Context(P=8, T=4096, D=4, k=1, B=1 << 15, rows=[8] * 4096, table_owner=[0] * 4096, part_kind=B.BLS_ROW_WISE)
    assert big.bls_sizes(0)["plan_ws_bytes"] > (1 << 20)
    with pytest.raises(B.BlsError) as e:                   # refused before anything touches a GPU
        big.bls_plan_noalloc(None, None, 0, None, None, None, None, None, None, None, 0)
    assert e.value.code == B.BLS_ENOSPC


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_missing_library_fails_loudly(B, monkeypatch, tmp_path):
    """No built library, no path: the binding raises instead of computing anything elsewhere."""
    import paper_2512_19342_amd.bls as mod
    monkeypatch.setattr(mod, "_lib", None)
    monkeypatch.setattr(mod, "lib_path", lambda: str(tmp_path / "libbls.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        mod.Context(2, 2, 4, 1, 4, [5, 5], [0, 1])


def test_product_never_imports_the_oracle():
    """The oracle is test infrastructure: nothing under the package or the generators names it."""
    import re
    for folder in ("paper_2512_19342_amd", "synth"):
        for dirpath, _, files in os.walk(os.path.join(ROOT, folder)):
            for f in files:
                if f.endswith((".py", ".hip", ".h", ".c", ".cpp")):
                    text = open(os.path.join(dirpath, f)).read()
                    assert not re.search(r"^\s*(import|from)\s+oracle\b", text, re.M), f
                    assert "bls_oracle" not in text and "orc_" not in text, f
