"""CPU-only checks of the boundary: the library loads, exports every declared symbol, and its host-side logic
(descriptor validation, arena sizing, argument checks that fire before any launch) behaves as documented.
No kernel is launched here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "kvq.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2604_04722_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build_library()
    return binding.load_library()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvq_[a-z0-9_]+)\s*\(", text)))


def test_every_symbol_declared_in_the_header_is_exported(lib):
    from paper_2604_04722_amd import binding
    names = declared_symbols()
    assert {"kvq_features", "kvq_controller", "kvq_append", "kvq_decode_attn"} <= set(names)
    for n in names:
        assert getattr(lib, n) is not None, n
    assert set(names) == set(binding.EXPORTED_SYMBOLS)


def test_header_compiles_as_plain_c(tmp_path):
    src = tmp_path / "t.c"
    src.write_text('#include "kvq.h"\nint main(void){kvq_cache_desc d; kvq_mlp m; (void)d; (void)m; return KVQ_OK;}\n')
    import subprocess
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                           "-c", str(src), "-o", str(tmp_path / "t.o")])


def make_desc(**kw):
    from paper_2604_04722_amd.binding import CacheDesc
    d = CacheDesc()
    d.n_layers, d.max_seqs, d.n_q_heads, d.n_kv_heads, d.head_dim = 24, 32, 32, 32, 64
    d.page_tokens, d.max_context = 0, 8192
    for k, v in kw.items():
        if k == "pool_pages":
            for c in range(4):
                d.pool_pages[c] = v[c]
        else:
            setattr(d, k, v)
    return d


def test_arena_size_follows_the_documented_block_sizes(lib):
    # pools dominate: layers * (pages+1 sink) * Hkv * blocks_per_page * block_bytes, block bytes 2560/4608/8704/16384
    pages = (20, 10, 6, 4)
    d = make_desc(pool_pages=pages)
    total = lib.kvq_cache_arena_bytes(ctypes.byref(d))
    pools = sum(24 * (p + 1) * 32 * 4 * bb for p, bb in zip(pages, (2560, 4608, 8704, 16384)))
    # bookkeeping per (sequence, position): the width (1 byte), its slot (4) and the slot -> position log (2 x 4)
    assert pools <= total <= pools + 32 * 8192 * 13 + (1 << 20)
    # per-token cost of a full block matches the algorithmic bytes per (token, kv-head): 40 / 72 / 136 / 256
    assert [bb // 64 for bb in (2560, 4608, 8704, 16384)] == [40, 72, 136, 256]


def test_default_pools_cover_the_worst_case(lib):
    d = make_desc(n_layers=1, max_seqs=2, n_q_heads=2, n_kv_heads=1, max_context=1000)
    total = lib.kvq_cache_arena_bytes(ctypes.byref(d))
    pages = 2 * 4                                           # max_seqs * ceil(1000/256)
    assert total >= sum((pages + 1) * 4 * bb for bb in (2560, 4608, 8704, 16384))


@pytest.mark.parametrize("kw", [dict(head_dim=128), dict(n_q_heads=30), dict(page_tokens=100), dict(max_context=0),
                                dict(n_layers=0), dict(pool_pages=(-1, 0, 0, 0)), dict(max_context=(1 << 26) + 1)])
def test_invalid_descriptors_are_rejected_on_the_host(lib, kw):
    d = make_desc(**kw)
    assert lib.kvq_cache_arena_bytes(ctypes.byref(d)) == 0
    assert lib.kvq_last_error().decode() != ""
    out = ctypes.c_void_p(None)
    assert lib.kvq_cache_create(ctypes.byref(d), ctypes.byref(out)) != 0
    assert not out.value


def test_null_and_range_checks_fire_before_any_launch(lib):
    from paper_2604_04722_amd.binding import Mlp
    assert lib.kvq_append(None, 0, None, None, None, None, 1, 1, None) == 1
    assert lib.kvq_decode_attn(None, 0, None, None, 1, None, None, None, None, 0, None) == 1
    assert lib.kvq_cache_reset(None, None) == 1
    assert lib.kvq_cache_destroy(None) == 0
    m = Mlp()
    m.n_linear = 4
    assert lib.kvq_controller(None, 1, ctypes.byref(m), None, None, None) == 3          # unsupported depth
    m.n_linear = 3
    m.dims[0], m.dims[1], m.dims[2], m.dims[3] = 4, 512, 16, 4
    assert lib.kvq_controller(None, 1, ctypes.byref(m), None, None, None) == 3          # hidden layer too wide
    m.dims[1] = 16
    m.dims[3] = 5
    assert lib.kvq_controller(None, 1, ctypes.byref(m), None, None, None) == 1          # not four classes
    assert lib.kvq_controller(None, -1, ctypes.byref(m), None, None, None) == 1
    assert lib.kvq_features(None, 1, 100, None, None, None, 0, None, None, None, 1, 0, None, None, 0, None) == 1
    assert lib.kvq_features(None, 0, 100, None, None, None, 0, None, None, None, 1, 0, None, None, 0, None) == 0   # n = 0
    assert lib.kvq_cache_set_length_hint(None, 5) == 1
    assert lib.kvq_tuning_set(b"no_such_entry", 1) == 1
    assert lib.kvq_tuning_set(b"attn_splits", 65) == 1
    assert lib.kvq_tuning_set(None, 1) == 1
    assert lib.kvq_features_workspace(32, 49152) >= 32 * 64 * 16
    assert b"kvq" in lib.kvq_version()


def test_launch_shape_table_round_trips_and_starts_from_the_environment(lib):
    """kvq_tuning_set / kvq_tuning_get on the host: defaults, a round trip, range checks that change nothing, and the
    KVQ_* environment variables as the table's starting values (read once, in a process of its own)."""
    import subprocess
    import sys
    v = ctypes.c_int32(-99)
    lib.kvq_tuning_get.argtypes = [ctypes.c_char_p, ctypes.POINTER(ctypes.c_int32)]
    lib.kvq_tuning_set.argtypes = [ctypes.c_char_p, ctypes.c_int32]
    defaults = {b"attn_splits": 0, b"attn_waves": 0, b"attn_longest_first": -1, b"attn_by_class": 12, b"append_bulk_min_T": 32,
                b"append_stream_min": 16, b"append_block_min_T": 512, b"controller_no_mfma": 0, b"train_no_mfma": 0}
    for name, want in defaults.items():
        assert lib.kvq_tuning_get(name, ctypes.byref(v)) == 0 and v.value == want, name
    assert lib.kvq_tuning_set(b"attn_splits", 7) == 0
    assert lib.kvq_tuning_get(b"attn_splits", ctypes.byref(v)) == 0 and v.value == 7
    assert lib.kvq_tuning_set(b"attn_splits", 65) == 1                       # out of range: refused, nothing changes
    assert lib.kvq_tuning_get(b"attn_splits", ctypes.byref(v)) == 0 and v.value == 7
    assert lib.kvq_tuning_set(b"attn_splits", 0) == 0
    assert lib.kvq_tuning_get(b"nope", ctypes.byref(v)) == 1 and lib.kvq_tuning_get(b"attn_splits", None) == 1
    code = ("import ctypes; l = ctypes.CDLL(%r); v = ctypes.c_int32(0); l.kvq_tuning_get(b'attn_splits', ctypes.byref(v)); a = v.value; "
            "l.kvq_tuning_get(b'attn_waves', ctypes.byref(v)); print(a, v.value)" % os.path.join(ROOT, "paper_2604_04722_amd", "libkvq.so"))
    env = dict(os.environ, KVQ_ATTN_SPLITS="3", KVQ_ATTN_WAVES="99")           # 99 is outside the entry's range: the default stays
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0 and r.stdout.split() == ["3", "0"], (r.stdout, r.stderr)


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    from paper_2604_04722_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(FileNotFoundError):
        binding.load_library()


def _sources(top):
    for dirpath, _, files in os.walk(os.path.join(ROOT, top)):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".c", ".cpp")):
                yield os.path.join(dirpath, f), open(os.path.join(dirpath, f)).read()


def test_product_and_oracle_never_import_each_other():
    """Neither tree names the other; the seeded input generators live in a package of their own that names neither."""
    for path, text in _sources("paper_2604_04722_amd"):
        assert "import oracle" not in text and "from oracle" not in text and "kvq_oracle" not in text, path
        assert "import workloads" not in text and "from workloads" not in text, path
    for path, text in _sources("oracle"):
        assert "paper_2604_04722_amd" not in text and "libkvq.so" not in text, path
    for path, text in _sources("workloads"):
        assert "paper_2604_04722_amd" not in text and "libkvq.so" not in text, path
        assert "import oracle" not in text and "from oracle" not in text and "kvq_oracle" not in text, path


def test_bench_refuses_more_than_one_gpu_before_touching_a_device():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
    assert r.stdout.strip() == ""                       # no JSON line for a run that did not happen
