"""Host-side checks that need no GPU: the shared library loads, exports every
symbol the header declares, validates arguments, and the accounting formulas
reproduce the paper's printed cache sizes."""
import ctypes
import os
import re

import pytest

import paper_2505_21487_amd as gla
from paper_2505_21487_amd import accounting

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "gla_decode.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(g[lqt]a_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = gla.load_library()
    names = header_functions()
    assert set(names) == set(gla.binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings():
    assert gla.gla_decode_version() >= 100
    seen = {gla.gla_status_string(c) for c in (0, -1, -2, -3, -4)}
    assert len(seen) == 5 and gla.gla_status_string(-99) == "unknown status"


def good(**over):
    kw = dict(batch=2, q_len=1, num_q_heads=16, num_groups=2, d_v=256, d_nope=256, d_rope=64,
              page_size=64, max_pages_per_seq=8, num_pages=100)
    kw.update(over)
    return gla.shape_params(**kw)


@pytest.mark.parametrize("over", [dict(q_len=0), dict(q_len=5), dict(num_groups=3), dict(d_nope=128),
                                  dict(page_size=0), dict(batch=-1), dict(num_splits=-1),
                                  dict(impl=7), dict(out_dtype=3), dict(d_v=0)])
def test_invalid_shapes_are_rejected_on_the_host(over):
    p = good(**over)
    assert gla.gla_decode_select_impl(p) == gla.GLA_ERR_INVALID_ARG
    assert gla.gla_decode_workspace_size(p) == 0
    assert gla.load_library().gla_decode(ctypes.byref(p)) == gla.GLA_ERR_INVALID_ARG


def test_gta_contract_on_d_nope():
    p = good(d_v=128, d_nope=64, num_q_heads=32, num_groups=4)
    assert gla.gla_decode_select_impl(p, True) > 0
    assert gla.gla_decode_select_impl(p, False) == gla.GLA_ERR_INVALID_ARG
    p = good(d_v=128, d_nope=128, num_q_heads=32, num_groups=4)
    assert gla.gla_decode_select_impl(p, True) == gla.GLA_ERR_INVALID_ARG


def test_null_pointers_and_missing_workspace_are_errors_not_launches():
    p = good(impl=gla.GLA_IMPL_GENERIC, num_splits=4)
    assert gla.load_library().gla_decode(ctypes.byref(p)) == gla.GLA_ERR_INVALID_ARG  # null q
    p.q_nope = p.q_rope = p.state_cache = p.rope_cache = 256   # never dereferenced on the host
    p.page_table = p.seq_lens = p.out = p.lse = 256
    assert gla.gla_decode_workspace_size(p) > 256
    assert gla.load_library().gla_decode(ctypes.byref(p)) == gla.GLA_ERR_WORKSPACE_TOO_SMALL
    p.workspace, p.workspace_bytes = 256, 16
    assert gla.load_library().gla_decode(ctypes.byref(p)) == gla.GLA_ERR_WORKSPACE_TOO_SMALL


def test_unsupported_shape_when_tuned_is_forced():
    p = good(d_v=96, d_nope=96, d_rope=32, page_size=16, impl=gla.GLA_IMPL_TUNED)
    assert gla.gla_decode_select_impl(p) == gla.GLA_ERR_UNSUPPORTED_SHAPE
    p.impl = gla.GLA_IMPL_AUTO
    assert gla.gla_decode_select_impl(p) == gla.GLA_IMPL_GENERIC


@pytest.mark.parametrize("page_size,tuned", [(64, True), (32, True), (16, True), (8, True), (4, True), (2, True),
                                             (1, True), (128, False), (48, False), (3, False)])
def test_page_sizes_the_tuned_kernel_takes(page_size, tuned):
    """Power-of-two pages up to 64 tokens have an MFMA instantiation for the three
    head shapes; anything else runs the generic kernel."""
    for kw, is_gta in ((dict(num_q_heads=128, num_groups=2, d_v=256, d_nope=256), False),
                       (dict(num_q_heads=128, num_groups=1, d_v=512, d_nope=512), False),
                       (dict(num_q_heads=32, num_groups=4, d_v=128, d_nope=64), True)):
        p = good(page_size=page_size, max_pages_per_seq=4096 // max(1, min(page_size, 64)), num_pages=100000, **kw)
        # dense layouts (strides take part in the choice; pointers stay null)
        h_q, h_c, d_v, d_n = kw["num_q_heads"], kw["num_groups"], kw["d_v"], kw["d_nope"]
        p.state_stride[:] = (h_c * page_size * d_v, page_size * d_v, d_v)
        p.rope_stride[:] = (page_size * 64, 64)
        p.q_nope_stride[:] = (h_q * d_n, h_q * d_n, d_n)
        p.q_rope_stride[:] = (h_q * 64, h_q * 64, 64)
        p.out_stride[:] = (h_q * d_v, h_q * d_v, d_v)
        p.softmax_scale = 0.05
        want = gla.GLA_IMPL_TUNED if tuned else gla.GLA_IMPL_GENERIC
        assert gla.gla_decode_select_impl(p, is_gta) == want
        assert gla.gla_decode_workspace_size(p, is_gta) > 0


def test_empty_batch_is_ok():
    p = good(batch=0)
    assert gla.load_library().gla_decode(ctypes.byref(p)) == gla.GLA_OK


# ---- accounting against the paper's printed numbers (tests/golden/*.txt)
def _rows(name):
    for line in open(os.path.join(ROOT, "tests", "golden", name)):
        line = line.strip()
        if line and not line.startswith("#"):
            yield line.split()


VARIANTS = {  # XL model of the paper: h_q = 16, d_h = 128
    "MHA": lambda tp: accounting.kv_bytes_per_token_heads(16, 128, 2, tp),
    "GQA-4": lambda tp: accounting.kv_bytes_per_token_heads(4, 128, 2, tp),
    "GTA-4": lambda tp: accounting.cache_bytes_per_token(4, 128, 64, tp),
    "GLA-2": lambda tp: accounting.cache_bytes_per_token(2, 256, 64, tp),
    "MLA": lambda tp: accounting.cache_bytes_per_token(1, 512, 64, tp),
}


def test_kv_bytes_per_token_match_the_papers_table():
    n = 0
    for name, tp, want in _rows("kv_bytes_per_token.txt"):
        assert VARIANTS[name](int(tp)) == int(want), (name, tp)
        n += 1
    assert n == 15


def test_per_device_cache_in_units_of_dh():
    d_h = 128
    f = {"MQA": lambda tp: accounting.kv_bytes_per_token_heads(1, d_h, 2, tp),
         "MLA": lambda tp: accounting.cache_bytes_per_token(1, 4 * d_h, d_h // 2, tp),
         "GLA-2": lambda tp: accounting.cache_bytes_per_token(2, 2 * d_h, d_h // 2, tp),
         "GTA-4": lambda tp: accounting.cache_bytes_per_token(8, d_h, d_h // 2, tp)}
    # the table's "GTA-4" row is the h_kv = 8 example of its caption: 8.5 d_h at TP = 1
    for row in _rows("kv_per_device_dh.txt"):
        name, vals = row[0], [float(v) for v in row[1:]]
        for tp, want in zip((1, 2, 4, 8), vals):
            assert f[name](tp) == want * d_h * 2, (name, tp)


def test_arithmetic_intensity_limits_of_table_1():
    L, h_q = 1e9, 128
    ai = accounting.paper_arithmetic_intensity
    assert abs(ai(L, h_q, h_q, 1) - 2 * h_q) < 1e-3          # MLA ~ 2 h_q
    assert abs(ai(L, h_q, h_q // 2, 1) - h_q) < 1e-3         # GLA-2 ~ h_q
    assert abs(ai(L, h_q, h_q, 2) - h_q) < 1e-3              # MQA ~ h_q
    assert abs(ai(L, h_q, 8, 2) - 8) < 1e-3                  # GQA ~ g_q
    assert abs(ai(L, h_q, 8, 1) - 16) < 1e-3                 # GTA ~ 2 g_q
    assert abs(ai(L, h_q, 1, 2) - 1) < 1e-3                  # MHA ~ 1
    # finite-L forms printed in the table
    L = 4096.0
    assert abs(ai(L, h_q, h_q // 2, 1) - L / (1 + L / h_q)) < 1e-9
    assert abs(ai(L, h_q, h_q, 1) - L / (1 + L / (2 * h_q))) < 1e-9


def test_counted_flops_per_byte_approach_the_papers_intensity():
    # GLA-2, h_q = 128, rope excluded: FLOPs / cache byte -> h_q as L grows
    L = [1 << 20]
    fl = accounting.flops(L, 1, 128, 256, 0, 256)
    by = accounting.cache_bytes(L, 2, 256, 0)
    assert abs(fl / by - 128) < 1e-6
    fl = accounting.flops(L, 1, 128, 512, 0, 512)
    by = accounting.cache_bytes(L, 1, 512, 0)
    assert abs(fl / by - 256) < 1e-6
    assert accounting.duplication_factor(2, 64, 128) == 1 and accounting.duplication_factor(4, 64, 128) == 2


# ---- the seeded workload generators the GPU tests and the benchmark draw from
@pytest.mark.parametrize("page_size", [64, 16, 1])
def test_workload_generators_build_consistent_problems(page_size):
    import workloads
    for p in (workloads.config(1, batch=2, max_len=300, page_size=page_size),
              workloads.config(4, batch=3, max_len=5000, page_size=page_size),
              workloads.latency_workload("100x2,700", shape="gla2", page_size=page_size),
              workloads.latency_workload("333", shape="mla", T=2, page_size=page_size)):
        assert p.page_size == page_size and p.num_pages == workloads.POOL_PAGES * 64 // page_size
        used = sum(-(-L // page_size) for L in p.seq_lens)
        assert len(p.page_ids) == used == len(set(int(x) for x in p.page_ids))
        for b, L in enumerate(p.seq_lens):          # every held table entry names a materialised page
            n = -(-L // page_size)
            assert set(int(x) for x in p.table_pool[b, :n]) <= set(int(x) for x in p.page_ids)
    assert workloads.parse_lens("1024x15,65536") == [1024] * 15 + [65536]


def test_register_page_windows_keep_their_registers():
    """The kernels that hold page-id windows in registers load them asynchronously
    from inline assembly; the compiler's output for them must name the same
    registers at every load site and write them nowhere else (a copy made while a
    load is in flight would carry stale page ids).  Cross-compiles the two
    kernels to assembly (no GPU needed, a few seconds) and checks exactly that."""
    from paper_2505_21487_amd import build

    found = build.check_register_windows(verbose=False)
    assert len(found) == 2


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: `bench.py --gpus N` with N above 1 (or a WORLD_SIZE above 1) exits with a message that says
    so, before anything touches a GPU."""
    import subprocess
    import sys

    for argv, env in ((["--gpus", "2"], {}), ([], {"WORLD_SIZE": "4"})):
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + argv, capture_output=True, text=True,
                           env=dict(os.environ, **env), timeout=120)
        assert r.returncode != 0
        assert "one GPU only" in (r.stdout + r.stderr)
