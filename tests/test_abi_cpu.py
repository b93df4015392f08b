"""Host-side logic of libtidal, no GPU needed: exported symbols, argument validation,
arena layout, the chunked copy plan.  No compute call is made."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2503_06421_amd import binding as tb
from paper_2503_06421_amd import workloads as wl_mod

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_ARENA = 0x7000_0000_0000          # never dereferenced by host-only calls


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(tb.LIB_PATH):
        from paper_2503_06421_amd import build
        build.build()
    tb.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "tidal.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tidal_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert len(names) >= 20
    L = ctypes.CDLL(tb.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n
    assert sorted(tb.EXPORTS) == names                       # the binding covers the same set


def test_config_defaults():
    c = tb.tidal_config_default()
    assert c.chunk_bytes == 128 << 20 and c.max_rank == 64 and c.coalesce_bytes == 64 << 10
    assert c.max_adapter_bytes == 0 and c.flags == 0


def test_required_bytes_and_slot_offsets(orc):
    shapes = [(3, 5), (1, 128), (7, 1), (128, 128), (0, 4), (1, 1)]
    cfg = tb.make_config(chunk_bytes=1 << 20, max_adapter_bytes=1000)
    need = tb.tidal_template_required_bytes(shapes, cfg)
    off = orc.layout(shapes)
    assert need == int(off[-1]) + 2 * (1 << 20) + 2 * 1024
    t = tb.tidal_template_create(shapes, FAKE_ARENA, need, cfg)
    try:
        for i, (r, c) in enumerate(shapes):
            p, n = tb.tidal_template_slot_ptr(t, i)
            assert p == FAKE_ARENA + int(off[i]) and n == 2 * r * c
    finally:
        tb.tidal_template_destroy(t)


def _expect(code, fn, *a, **k):
    with pytest.raises(tb.TidalError) as e:
        fn(*a, **k)
    assert e.value.code == code, str(e.value)
    assert tb.tidal_last_error()
    return str(e.value)


def test_create_rejects_bad_arguments():
    shapes = [(4, 4)]
    need = tb.tidal_template_required_bytes(shapes)
    _expect(tb.TIDAL_E_NOMEM, tb.tidal_template_create, shapes, FAKE_ARENA, need - 1)
    _expect(tb.TIDAL_E_INVAL, tb.tidal_template_create, shapes, FAKE_ARENA + 8, need)
    _expect(tb.TIDAL_E_INVAL, tb.tidal_template_create, shapes, 0, need)
    _expect(tb.TIDAL_E_INVAL, tb.tidal_template_create, [(-1, 4)], FAKE_ARENA, need)
    for bad in (tb.make_config(chunk_bytes=1024), tb.make_config(max_rank=65), tb.make_config(flags=256),
                tb.make_config(chunk_bytes=1 << 20, coalesce_bytes=1 << 21)):
        _expect(tb.TIDAL_E_INVAL, tb.tidal_template_create, shapes, FAKE_ARENA, 1 << 40, bad)
        assert tb.tidal_template_required_bytes(shapes, bad) == 0


@pytest.fixture()
def small_template():
    shapes = [(8, 16), (4, 4), (1, 32)]
    cfg = tb.make_config(max_adapter_bytes=1 << 16)
    t = tb.tidal_template_create(shapes, FAKE_ARENA, 1 << 40, cfg)
    yield t, shapes
    tb.tidal_template_destroy(t)


def test_validation_happens_before_any_device_work(small_template):
    t, shapes = small_template
    a = np.zeros((8, 16), np.float32)
    _expect(tb.TIDAL_E_INVAL, tb.tidal_materialize, t, [(3, tb.TIDAL_F32, a.ctypes.data)])
    _expect(tb.TIDAL_E_INVAL, tb.tidal_materialize, t, [(0, 7, a.ctypes.data)])
    _expect(tb.TIDAL_E_INVAL, tb.tidal_materialize, t, [(0, tb.TIDAL_F32, None)])
    _expect(tb.TIDAL_E_INVAL, tb.tidal_materialize, t, [(0, tb.TIDAL_F32, a.ctypes.data)] * 2)
    A = np.zeros((2, 16), np.float32)
    B = np.zeros((8, 2), np.float32)
    ok = (0, 2, 4.0, tb.TIDAL_F32, A.ctypes.data, B.ctypes.data)
    _expect(tb.TIDAL_E_INVAL, tb.tidal_lora_attach, t, [(5,) + ok[1:]])
    _expect(tb.TIDAL_E_INVAL, tb.tidal_lora_attach, t, [(0, 65) + ok[2:]])
    _expect(tb.TIDAL_E_INVAL, tb.tidal_lora_attach, t, [(0, -1) + ok[2:]])
    _expect(tb.TIDAL_E_INVAL, tb.tidal_lora_attach, t, [ok, ok])
    _expect(tb.TIDAL_E_INVAL, tb.tidal_lora_attach, t, [(0, 2, 4.0, 9, A.ctypes.data, B.ctypes.data)])
    _expect(tb.TIDAL_E_INVAL, tb.tidal_lora_attach, t, [(0, 2, 4.0, tb.TIDAL_F32, None, B.ctypes.data)])
    _expect(tb.TIDAL_E_INVAL, tb.tidal_lora_attach, t, [(0, 2, float("nan"), tb.TIDAL_F32, A.ctypes.data, B.ctypes.data)])
    # state errors that need no device: nothing attached, slot never materialised
    _expect(tb.TIDAL_E_STATE, tb.tidal_lora_swap, t, [ok])
    _expect(tb.TIDAL_E_STATE, tb.tidal_lora_detach, t)
    _expect(tb.TIDAL_E_STATE, tb.tidal_lora_attach, t, [ok])
    _expect(tb.TIDAL_E_STATE, tb.tidal_template_slot_wait, t, 0)
    # A transposed (16 columns padded to a strip of 256, 16 ranks) + B (8 rows padded to a block of 32)
    # + row-major A (2 x 16 -> one 256-byte unit)
    assert tb.tidal_adapter_required_bytes(t, [ok]) == 2 * 256 * 16 + 2 * 32 * 16 + 256
    assert tb.tidal_adapter_required_bytes(t, [(9,) + ok[1:]]) == 0


def test_adapter_too_large_for_region():
    shapes = [(64, 64)]
    cfg = tb.make_config(max_adapter_bytes=256)
    t = tb.tidal_template_create(shapes, FAKE_ARENA, 1 << 40, cfg)
    try:
        A = np.zeros((4, 64), np.float32)
        B = np.zeros((64, 4), np.float32)
        # the size check comes after the materialised check, so look at the size directly
        assert tb.tidal_adapter_required_bytes(t, [(0, 4, 8.0, tb.TIDAL_F32, A.ctypes.data, B.ctypes.data)]) == 2 * 256 * 16 + 2 * 64 * 16 + 512
    finally:
        tb.tidal_template_destroy(t)


def test_factor_larger_than_a_chunk_is_rejected_up_front():
    """A factor is staged whole; one that cannot fit a staging buffer is an argument error of the call,
    found before anything is enqueued (also when another target comes first)."""
    shapes = [(8, 16), (64, 40000)]
    cfg = tb.make_config(chunk_bytes=64 << 10, max_adapter_bytes=1 << 24)
    t = tb.tidal_template_create(shapes, FAKE_ARENA, 1 << 40, cfg)
    try:
        a0, b0 = np.zeros((2, 16), np.float32), np.zeros((8, 2), np.float32)
        A, B = np.zeros((1, 40000), np.float32), np.zeros((64, 1), np.float32)     # A: 160,000 bytes > 65,536
        small = (0, 2, 4.0, tb.TIDAL_F32, a0.ctypes.data, b0.ctypes.data)
        big = (1, 1, 2.0, tb.TIDAL_F32, A.ctypes.data, B.ctypes.data)
        with pytest.raises(tb.TidalError) as e:
            tb.tidal_lora_attach(t, [small, big])
        assert e.value.code == tb.TIDAL_E_INVAL and "chunk_bytes" in str(e.value)
        half = (1, 1, 2.0, tb.TIDAL_F16, A.ctypes.data, B.ctypes.data)             # 80,000 bytes: still too large
        _expect(tb.TIDAL_E_INVAL, tb.tidal_lora_attach, t, [half])
    finally:
        tb.tidal_template_destroy(t)


def _check_plan(plan, shapes, dtypes, chunk_bytes, coalesce, pinned):
    isz = {tb.TIDAL_F32: 4, tb.TIDAL_F16: 2, tb.TIDAL_BF16: 2}
    # every element of every slot is covered exactly once, in order
    pos = {}
    last_chunk = 0
    order = []
    for p in plan:
        assert p.chunk >= last_chunk
        last_chunk = p.chunk
        assert p.elem_offset == pos.get(p.slot, 0)
        pos[p.slot] = p.elem_offset + p.elems
        assert p.src_bytes == p.elems * isz[dtypes[p.slot]]
        if not order or order[-1] != p.slot:
            order.append(p.slot)
        staged = dtypes[p.slot] != tb.TIDAL_BF16
        assert (p.staging_offset >= 0) == staged
        if staged:
            assert p.staging_offset % 256 == 0
            assert p.staging_offset + p.src_bytes <= chunk_bytes
            assert p.elem_offset % 128 == 0
        small = shapes[p.slot][0] * shapes[p.slot][1] * isz[dtypes[p.slot]] < coalesce
        assert bool(p.gathered) == (small or not pinned)
    for s, (r, c) in enumerate(shapes):
        assert pos.get(s, 0) == r * c
    assert order == [s for s in range(len(shapes)) if shapes[s][0] * shapes[s][1] > 0]
    # staged pieces of one chunk do not overlap and stay below the segment limit
    by_chunk = {}
    for p in plan:
        if p.staging_offset >= 0:
            by_chunk.setdefault(p.chunk, []).append((p.staging_offset, p.staging_offset + p.src_bytes))
    for spans in by_chunk.values():
        assert len(spans) <= 32
        spans.sort()
        for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
            assert a1 <= b0


@pytest.mark.parametrize("pinned", [1, 0])
@pytest.mark.parametrize("dtype", [tb.TIDAL_F32, tb.TIDAL_F16, tb.TIDAL_BF16])
def test_copy_plan_covers_everything_once(pinned, dtype):
    w = wl_mod.tiny_stack(with_norms=True, layers=3, hidden=320, ffn=872, vocab=3000)
    shapes = w.shapes + [(0, 7), (1, 1), (3, 43)]
    chunk = 256 << 10
    cfg = tb.make_config(chunk_bytes=chunk, coalesce_bytes=4096)
    t = tb.tidal_template_create(shapes, FAKE_ARENA, 1 << 40, cfg)
    try:
        dtypes = [dtype] * len(shapes)
        srcs = [(i, dtype, 0x1000 + 16 * i) for i in range(len(shapes))]
        plan = tb.tidal_materialize_plan(t, srcs, assume_pinned=pinned)
        _check_plan(plan, shapes, dtypes, chunk, 4096, bool(pinned))
        n_chunks = plan[-1].chunk + 1
        total = sum(p.src_bytes for p in plan)
        if dtype != tb.TIDAL_BF16 or not pinned:
            assert n_chunks <= -(-total // chunk) + sum(1 for s in shapes if s[0] * s[1]) // 32 + 2
            # small tensors never get a chunk of their own (tensor merging)
            small = {i for i, sh in enumerate(shapes) if 0 < sh[0] * sh[1] * 4 <= 4096}
            alone = [p for p in plan if p.slot in small and sum(q.chunk == p.chunk for q in plan) == 1]
            assert small and not alone
    finally:
        tb.tidal_template_destroy(t)


def test_copy_plan_llama7b_chunk_count():
    """Tensor merging at scale: 226 tensors / 13.48 GB of fp16 become ~200 uniform chunks."""
    w = wl_mod.llama2_7b()
    t = tb.tidal_template_create(w.shapes, FAKE_ARENA, 1 << 40, None)
    try:
        srcs = [(i, tb.TIDAL_F16, 0x1000) for i in range(len(w.shapes))]
        plan = tb.tidal_materialize_plan(t, srcs, assume_pinned=1)
        assert sum(p.src_bytes for p in plan) == w.source_bytes
        assert plan[-1].chunk + 1 == -(-w.source_bytes // (128 << 20))     # every chunk full but the last
        assert not any(p.gathered for p in plan)
    finally:
        tb.tidal_template_destroy(t)


def test_no_device_means_error_not_fallback(small_template):
    """On a host without a GPU the data path reports TIDAL_E_HIP; it never computes on the CPU."""
    try:
        import torch
        if torch.cuda.is_available():
            pytest.skip("GPU present")
    except ImportError:
        pass
    t, shapes = small_template
    a = np.zeros((8, 16), np.float32)
    _expect(tb.TIDAL_E_HIP, tb.tidal_materialize, t, [(0, tb.TIDAL_F32, a.ctypes.data)])


def test_prefetch_rule_and_resident_prefix_match_oracle(orc):
    """Eq. 1 of the paper's Sec. 5.2 and the slot-granular prefix that realises it (host-only)."""
    cases = [(24_300_000_000, 0.4, 32e9), (24_300_000_000, 1.0, 32e9), (13_476_298_752, 0.12, 57.3e9),
             (1000, 1e-9, 1e9), (1000, 0.5e-9, 1e9), (0, 1.0, 1.0), (5, 0.0, 0.0)]
    for m, tt, bw in cases:
        assert tb.tidal_prefetch_bytes(m, tt, bw) == orc.prefetch_bytes(m, tt, bw), (m, tt, bw)
    assert tb.tidal_prefetch_bytes(100, -1.0, 1.0) == 0 and tb.tidal_prefetch_bytes(100, float("nan"), 1.0) == 0
    w = wl_mod.llama2_7b()
    t = tb.tidal_template_create(w.shapes, FAKE_ARENA, 1 << 40, None)
    try:
        for pre in (0, 1, 262_144_000, 262_144_001, 5_000_000_000, w.source_bytes, w.source_bytes + 1):
            n, b = tb.tidal_template_resident_prefix(t, pre)
            assert n == orc.resident_prefix(w.shapes, pre)
            assert b == sum(2 * r * c for r, c in w.shapes[:n])
            assert b >= min(pre, w.source_bytes)
    finally:
        tb.tidal_template_destroy(t)


def test_copy_plan_property_fuzz():
    """Random slot lists, dtypes, chunk sizes, coalescing thresholds and pinned-ness: the plan always
    covers every element once, in order, within the buffer limits (hypothesis)."""
    hyp = pytest.importorskip("hypothesis")
    st = hyp.strategies

    @hyp.settings(max_examples=150, deadline=None)
    @hyp.given(shapes=st.lists(st.tuples(st.integers(0, 700), st.integers(0, 900)), min_size=1, max_size=24),
               dtype=st.sampled_from([tb.TIDAL_F32, tb.TIDAL_F16, tb.TIDAL_BF16]),
               chunk_kib=st.integers(64, 512), coalesce_log=st.integers(0, 16), pinned=st.booleans(),
               skip=st.integers(0, 5))
    def run(shapes, dtype, chunk_kib, coalesce_log, pinned, skip):
        chunk = -(-(chunk_kib << 10) // 4096) * 4096
        coalesce = 1 << coalesce_log
        cfg = tb.make_config(chunk_bytes=chunk, coalesce_bytes=coalesce)
        t = tb.tidal_template_create(shapes, FAKE_ARENA, 1 << 40, cfg)
        try:
            used = [i for i in range(len(shapes)) if (i + skip) % 6 != 0]
            srcs = [(i, dtype, 0x1000 + 64 * i) for i in used]
            plan = tb.tidal_materialize_plan(t, srcs, assume_pinned=int(pinned))
            sub = [shapes[i] if i in used else (0, 0) for i in range(len(shapes))]
            if any(r * c for r, c in sub):
                _check_plan(plan, sub, [dtype] * len(shapes), chunk, coalesce, pinned)
            else:
                assert plan == []
        finally:
            tb.tidal_template_destroy(t)

    run()


def test_lora_apply_validates_segments_without_a_device():
    t = tb.tidal_template_create([(64, 64)], FAKE_ARENA, 1 << 40, tb.make_config())
    try:
        assert tb.tidal_lora_apply_workspace_bytes(0) == 256
        assert tb.tidal_lora_apply_workspace_bytes(3) == 512            # 3 tokens x 64 ranks x 2 bytes, 256-aligned
        # no adapters: segments without an adapter are a no-op that needs no device
        tb.tidal_lora_apply(t, 0, [], [(-1, 0, 4)], 0, 0, 8, 0, 0)
        _expect(tb.TIDAL_E_INVAL, tb.tidal_lora_apply, t, 0, [], [(-1, 0, 5), (-1, 4, 8)], 0, 0, 8, 0, 0)
        _expect(tb.TIDAL_E_INVAL, tb.tidal_lora_apply, t, 0, [], [(-1, 0, 9)], 0, 0, 8, 0, 0)
        _expect(tb.TIDAL_E_INVAL, tb.tidal_lora_apply, t, 0, [], [(0, 0, 4)], 0, 0, 8, 0, 0)
        _expect(tb.TIDAL_E_INVAL, tb.tidal_lora_apply, t, 1, [], [], 0, 0, 8, 0, 0)
        _expect(tb.TIDAL_E_INVAL, tb.tidal_lora_apply, t, 0, [], [], 0, 0, -1, 0, 0)
    finally:
        tb.tidal_template_destroy(t)


def test_gather_threads_default_and_range():
    cfg = tb.tidal_config_default()
    assert cfg.gather_threads == 4
    assert tb.tidal_template_required_bytes([(4, 4)], tb.make_config(gather_threads=16)) > 0
    assert tb.tidal_template_required_bytes([(4, 4)], tb.make_config(gather_threads=17)) == 0
    assert tb.tidal_template_required_bytes([(4, 4)], tb.make_config(gather_threads=-1)) == 0


def test_chunks_ahead_default_and_range():
    assert tb.tidal_config_default().chunks_ahead == 160                      # 128 MiB chunks
    for kw in (dict(chunks_ahead=1), dict(chunks_ahead=4096), dict(chunk_bytes=1 << 20)):
        assert tb.tidal_template_required_bytes([(4, 4)], tb.make_config(**kw)) > 0
    assert tb.tidal_template_required_bytes([(4, 4)], tb.make_config(chunks_ahead=4097)) == 0
    assert tb.tidal_template_required_bytes([(4, 4)], tb.make_config(chunks_ahead=-1)) == 0


def test_header_is_plain_c_and_links_from_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 (and C++), and a C program must
    link against the library and call a host-only entry point."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "use_tidal.c"
    src.write_text(
        '#include <stdio.h>\n#include "tidal.h"\n'
        'int main(void) {\n'
        '    tidal_config c; tidal_slot_desc s[2] = {{4, 8}, {3, 5}};\n'
        '    if (tidal_config_default(&c) != TIDAL_OK) return 1;\n'
        '    size_t need = tidal_template_required_bytes(s, 2, &c);\n'
        '    tidal_template* t = 0;\n'
        '    if (tidal_template_create(s, 2, (void*)0x700000000000ull, need, &c, &t) != TIDAL_OK) return 2;\n'
        '    if (tidal_prefetch_bytes(1000, 0.5, 1000.0) != 500) return 3;\n'
        '    printf("%zu %s\\n", need, tidal_last_error());\n'
        '    return tidal_template_destroy(t);\n}\n')
    inc = os.path.join(root, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, "-c", str(src), "-o",
                    str(tmp_path / "c.o")], check=True)
    subprocess.run(["g++", "-std=c++11", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, "-x", "c++", "-c", str(src),
                    "-o", str(tmp_path / "cxx.o")], check=True)
    libdir = os.path.dirname(tb.LIB_PATH)
    exe = tmp_path / "use_tidal"
    subprocess.run(["gcc", str(tmp_path / "c.o"), "-o", str(exe), "-L", libdir, "-ltidal", "-Wl,-rpath," + libdir],
                   check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert int(out[0]) == tb.tidal_template_required_bytes([(4, 8), (3, 5)])


# ---- groups of the adapter upload (tidal_lora_attach / _swap with host pointers) ---------------------

def _fake_targets(wl, r, dtype):
    """Targets with host addresses that are never read (the plan only looks at sizes)."""
    return [(s, r, 2.0 * r, dtype, 0x10000 + 64 * k, 0x20000 + 64 * k) for k, s in enumerate(wl.lora_slots)]


def _raw_bytes(wl, slots, r, itemsize):
    return sum(r * (wl.tensors[s].rows + wl.tensors[s].cols) * itemsize for s in slots)


def test_upload_plan_of_the_listed_workloads():
    """Default rates (55 GB/s link, 6 TB/s pass).  A merge-bound adapter gets a small first group and
    growing later ones; an upload-bound one many near-equal groups; no group exceeds half the staging span."""
    half_span = 128 << 20
    seen = {}
    for name, dt, isz in (("llama2_7b", tb.TIDAL_F16, 2), ("llama2_13b", tb.TIDAL_F16, 2), ("llama3_70b", tb.TIDAL_BF16, 2)):
        wl = getattr(wl_mod, name)()
        t = tb.tidal_template_create(wl.shapes, FAKE_ARENA, 1 << 40, tb.make_config())
        try:
            g = tb.tidal_lora_upload_plan(t, _fake_targets(wl, wl.rank, dt))
            assert g == tb.tidal_lora_upload_plan(t, _fake_targets(wl, wl.rank, dt), swap=True)   # nothing attached
        finally:
            tb.tidal_template_destroy(t)
        assert sum(g) == len(wl.lora_slots) and all(x > 0 for x in g) and 2 <= len(g) <= 8, (name, g)
        a = 0
        for x in g:
            assert _raw_bytes(wl, wl.lora_slots[a:a + x], wl.rank, isz) <= half_span, (name, g)
            a += x
        seen[name] = g
    # 7B: merges take twice the upload -> three groups, each about twice the one before
    assert len(seen["llama2_7b"]) == 3 and seen["llama2_7b"][0] <= 12 and seen["llama2_7b"] == sorted(seen["llama2_7b"])
    # 13B: upload and merges take the same time -> as many groups as there may be, equal but for a smaller first
    g = seen["llama2_13b"]
    assert len(g) == 8 and max(g[1:]) - min(g[1:]) <= 4 and g[0] <= g[1]
    # 70B: merges take six times the upload -> a first group of a few megabytes, steep growth, capped by the span
    g = seen["llama3_70b"]
    assert len(g) <= 6 and g[0] <= 16 and g[1] >= 3 * g[0] and max(g) >= 150


def test_upload_plan_single_group_cases_and_flags():
    wl = wl_mod.llama2_7b()
    tg = _fake_targets(wl, 16, tb.TIDAL_F16)
    n = len(tg)
    cases = [
        (tb.make_config(flags=tb.TIDAL_FLAG_SERIAL_UPLOAD), tg, [n]),            # grouping forbidden
        (tb.make_config(), tg[:1], [1]),                                          # one target
        (tb.make_config(), tg[:8], [8]),                                          # 2 MiB of factors: below 4 MiB
        (tb.make_config(chunk_bytes=1 << 20), tg, [n]),                           # no split into <= 8 groups fits 1 MiB each
    ]
    for cfg, targets, want in cases:
        t = tb.tidal_template_create(wl.shapes, FAKE_ARENA, 1 << 40, cfg)
        try:
            assert tb.tidal_lora_upload_plan(t, targets) == want
        finally:
            tb.tidal_template_destroy(t)
    # forced grouping of a small adapter; idle targets (rank 0) ride along in whatever group they fall into
    t = tb.tidal_template_create(wl.shapes, FAKE_ARENA, 1 << 40, tb.make_config(flags=tb.TIDAL_FLAG_PIPELINED_UPLOAD))
    try:
        g = tb.tidal_lora_upload_plan(t, tg[:8])
        assert len(g) >= 2 and sum(g) == 8
        mixed = [(s, 0, 1.0, tb.TIDAL_F32, None, None) if k % 3 == 0 else x for k, (x, s) in enumerate(zip(tg, wl.lora_slots))]
        g = tb.tidal_lora_upload_plan(t, mixed)
        assert sum(g) == n and all(x > 0 for x in g)
        # argument checks are those of the attach
        _expect(tb.TIDAL_E_INVAL, tb.tidal_lora_upload_plan, t, [(wl.lora_slots[0], 65, 1.0, tb.TIDAL_F16, 0x1000, 0x2000)])
        _expect(tb.TIDAL_E_INVAL, tb.tidal_lora_upload_plan, t, [tg[0], tg[0]])
        _expect(tb.TIDAL_E_INVAL, tb.tidal_lora_upload_plan, t, [(10 ** 6, 8, 1.0, tb.TIDAL_F16, 0x1000, 0x2000)])
    finally:
        tb.tidal_template_destroy(t)


def test_upload_plan_properties_on_random_stacks():
    rng = np.random.default_rng(5)
    for case in range(40):
        n = int(rng.integers(2, 200))
        dims = [int(rng.choice([1024, 2048, 4096, 5120, 8192, 11008])) for _ in range(2)]
        shapes = [(dims[k % 2], dims[(k + 1) % 2]) for k in range(n)]
        r = int(rng.choice([4, 8, 16, 32, 64]))
        chunk = int(rng.choice([8, 32, 128])) << 20
        t = tb.tidal_template_create(shapes, FAKE_ARENA, 1 << 42, tb.make_config(chunk_bytes=chunk))
        try:
            tg = [(k, r, 1.0, tb.TIDAL_F16, 0x1000, 0x2000) for k in range(n)]
            g = tb.tidal_lora_upload_plan(t, tg)
        finally:
            tb.tidal_template_destroy(t)
        assert sum(g) == n and all(x > 0 for x in g) and len(g) <= 8, (case, g)
        if len(g) > 1:
            a = 0
            for x in g:
                raw = sum(r * (shapes[k][0] + shapes[k][1]) * 2 + 512 for k in range(a, a + x))
                assert raw <= chunk, (case, g)                           # half the span of two staging buffers
                a += x
