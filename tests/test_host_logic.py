"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, validates
arguments, fails loudly without a GPU, and its host-side page allocator keeps its books."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2506_06122_amd as R
from paper_2506_06122_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "rollout.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rollout_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = R.load_library()
    names = declared_symbols()
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), f"{n} declared in rollout.h but not exported"
    assert set(names) == set(B.SIGNATURES), "binding and header disagree on the entry points"
    assert lib.rollout_abi_version() == 3


def test_init_validates_and_fails_loudly_without_gpu():
    lib = R.load_library()
    layers = (B.rollout_layer_weights * 2)()
    w = B.rollout_weights(1, 1, 1, layers)
    rd = B.rollout_runtime_desc(1 << 20, 32, 8, 128, 256, None, 0, 0, 0)
    ctx = C.c_void_p()

    def init(**over):
        f = dict(n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn_dim=688, vocab=1024,
                 n_experts=0, top_k=0, expert_ffn_dim=0, rms_eps=1e-6, rope_theta=1e4, dtype=0, flags=0)
        f.update(over)
        md = B.rollout_model_desc(*f.values())
        rc = lib.rollout_init(C.byref(ctx), C.byref(md), C.byref(w), C.byref(rd))
        return rc, lib.rollout_last_error(None).decode()

    assert init(head_dim=30)[0] == B.E_INVAL
    assert init(n_q_heads=3)[0] == B.E_INVAL
    assert init(dtype=7)[0] == B.E_INVAL
    assert init(flags=8)[0] == B.E_INVAL          # 1, 2, 4 are the model-family options
    assert init(n_experts=4, top_k=5, expert_ffn_dim=8)[0] == B.E_INVAL
    rd.page_tokens = 24
    assert init()[0] == B.E_INVAL
    rd.page_tokens = 32
    assert lib.rollout_init(None, None, None, None) == B.E_INVAL
    import torch
    if not torch.cuda.is_available():
        rc, msg = init()
        assert rc == B.E_HIP and "HIP" in msg and not ctx.value    # no silent CPU path


def test_null_context_is_rejected():
    lib = R.load_library()
    n = C.c_int32(4)
    assert lib.rollout_decode_step(None, None, None, C.byref(n), None, None, None, None) == B.E_INVAL
    assert lib.rollout_abort(None, 0, None) == B.E_INVAL
    assert lib.rollout_logprobs(None, 0, None, None, 1.0, None) == B.E_INVAL
    assert lib.rollout_live_samples(None, 0, None) == B.E_INVAL
    lib.rollout_destroy(None)


# ------------------------------------------------------------------ page pool
def test_pool_alloc_release_and_refcounts():
    p = R.PagePool(5)
    pages = [p.alloc() for _ in range(5)]
    assert sorted(pages) == [0, 1, 2, 3, 4] and p.free_pages() == 0
    assert p.alloc() == B.E_NOMEM
    assert p.retain(pages[0]) == 2 and p.refcount(pages[0]) == 2
    assert p.release(pages[0]) == 1 and p.free_pages() == 0
    assert p.release(pages[0]) == 0 and p.free_pages() == 1
    assert p.release(pages[0]) == B.E_INVAL                 # never negative
    assert p.retain(pages[0]) == B.E_INVAL and p.retain(99) == B.E_INVAL
    for q in pages[1:]:
        assert p.release(q) == 0
    assert p.free_pages() == 5 and all(p.refcount(q) == 0 for q in pages)


def test_pool_reservations_are_honoured():
    p = R.PagePool(6)
    assert p.reserve(4) == B.OK and p.unreserved() == 2
    assert p.reserve(3) == B.E_NOMEM and p.unreserved() == 2
    a, b = p.alloc(False), p.alloc(False)
    assert a >= 0 and b >= 0 and p.alloc(False) == B.E_NOMEM     # the rest is promised
    got = [p.alloc(True) for _ in range(4)]
    assert all(g >= 0 for g in got) and p.alloc(True) == B.E_NOMEM
    p.unreserve(10)
    assert p.unreserved() == 0 and p.free_pages() == 0


def test_pool_random_walk_conserves_pages():
    rng = np.random.default_rng(0)
    p = R.PagePool(64)
    held = {}
    for _ in range(5000):
        op = rng.integers(0, 3)
        if op == 0:
            pg = p.alloc()
            if pg >= 0:
                assert pg not in held
                held[pg] = 1
            else:
                assert len(held) == 64
        elif op == 1 and held:
            pg = int(rng.choice(list(held)))
            held[pg] += 1
            assert p.retain(pg) == held[pg]
        elif held:
            pg = int(rng.choice(list(held)))
            held[pg] -= 1
            assert p.release(pg) == held[pg]
            if not held[pg]:
                del held[pg]
        assert p.free_pages() == 64 - len(held)
    for pg, n in list(held.items()):
        for _ in range(n):
            p.release(pg)
    assert p.free_pages() == 64


@pytest.mark.parametrize("prompt_len,page,max_new", [(70, 32, [1, 2, 40]), (64, 32, [1, 2, 33, 34]),
                                                       (5, 32, [1, 28, 29]), (512, 64, [2048] * 8)])
def test_plan_pages_matches_direct_count(prompt_len, page, max_new):
    total, shared, tail, priv = R.rollout_plan_pages(prompt_len, page, max_new)
    assert shared == prompt_len // page and tail == int(prompt_len % page != 0)
    for m, got in zip(max_new, priv):
        if m == 1:
            assert got == 0                                  # never decodes, holds nothing
            continue
        cached = set(range(prompt_len + m - 1))              # positions that end up in the cache
        own = {pos // page for pos in cached} - set(range(shared))
        assert got == len(own)
    assert total == shared + tail + int(priv.sum())


def test_bench_step_trace_table(tmp_path):
    """bench.py's per-step table: bins cover every decode step once, the live-sample counts it
    derives from the load must equal the ones the calls reported."""
    import bench
    import workloads
    load = workloads.load_c2(n_prompts=3)
    new = load.max_new_tokens.astype(np.int64)
    trace = [(0, 0.05)] + [(int((new > t).sum()), 1e-3) for t in range(1, int(new.max()))]
    out = tmp_path / "trace.txt"
    bench.write_step_trace(str(out), trace, load, 28 * 1024, 3_000_000_000, "python bench.py --step-trace x")
    lines = out.read_text().splitlines()
    assert lines[1] == "command: python bench.py --step-trace x"
    rows = [l.split() for l in lines[4:]]
    assert sum(int(r[1]) for r in rows) == len(trace) - 1
    assert abs(sum(float(r[-2]) for r in rows) - 100.0) < 0.5
    with pytest.raises(AssertionError):   # a step whose count disagrees with the load's lengths
        bench.write_step_trace(str(out), trace[:5] + [(trace[5][0] + 1, 1e-3)] + trace[6:], load, 1, 1, "x")
