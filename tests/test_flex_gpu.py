"""GPU parity of the head shapes served by the second MFMA kernel: small tied
states (GTA with d_h 64 / 96, RoPE key d_h / 2), latent heads of 128 dims, and
the grouped-query baseline with separate key / value caches, against the CPU
oracle.  impl = TUNED must find an MFMA kernel for every one of them."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_21487_amd as gla
from paper_2505_21487_amd.harness import DeviceProblem
from workloads import config, make_problem, uniform_lengths

from gpu_util import check_problem

pytestmark = pytest.mark.gpu

GENERIC, TUNED = gla.GLA_IMPL_GENERIC, gla.GLA_IMPL_TUNED
LENS = [0, 1, 31, 32, 33, 63, 64, 65, 130, 700, 1500, 2600]

SHAPES = {
    "gta64": dict(kind="gta", h_q=32, h_c=4, d_v=64, d_r=32),
    "gta96": dict(kind="gta", h_q=24, h_c=4, d_v=96, d_r=48),
    "gla128": dict(kind="gla", h_q=32, h_c=2, d_v=128, d_r=32),
    "gqa128": dict(kind="gqa", h_q=32, h_c=4, d_v=128),
    "gqa64": dict(kind="gqa", h_q=16, h_c=8, d_v=64),
}


def mfma_kernel_selected(p):
    prm = gla.shape_params(batch=p.B, q_len=p.T, num_q_heads=p.h_q, num_groups=p.h_c, d_v=p.d_v, d_nope=p.d_n,
                           d_rope=p.d_r, page_size=p.page_size, max_pages_per_seq=p.max_pages, num_pages=p.num_pages,
                           impl=TUNED)
    prm.softmax_scale = p.scale
    prm.state_stride = (p.h_c * p.page_size * p.d_v, p.page_size * p.d_v, p.d_v)
    prm.rope_stride = (p.page_size * p.d_r, p.d_r)
    return gla.gla_decode_select_impl(prm, {"gla": 0, "gta": 1, "gqa": 2}[p.kind]) == TUNED


@pytest.mark.parametrize("T", [1, 2, 4])
@pytest.mark.parametrize("page_size", [64, 32])
@pytest.mark.parametrize("shape", list(SHAPES))
def test_small_head_shapes(shape, page_size, T):
    p = make_problem(f"flex_{shape}", seq_lens=LENS, T=T, page_size=page_size, num_pages=4096, seed=1100 + 7 * T + page_size,
                     poison_tail=True, extra_table_cols=1, **SHAPES[shape])
    assert mfma_kernel_selected(p)
    for impl in (TUNED, GENERIC):
        check_problem(p, impl=impl, what=f"{shape} page {page_size} T={T} impl={impl}")


@pytest.mark.parametrize("page_size", [16, 8, 2, 1])
@pytest.mark.parametrize("shape", list(SHAPES))
def test_small_pages(shape, page_size):
    """Pages of fewer than 32 tokens: a tile spans 2 to 32 pages, every lane forms
    the address of its row from that row's page id; sequences long enough to move
    the wave's 64 held page ids many times, with the automatic split and as one
    chunk per sequence, T = 1 and 3."""
    for T, splits in ((1, 0), (3, 1), (2, 5)):
        p = make_problem(f"flex_sp_{shape}", seq_lens=LENS + [4100], T=T, page_size=page_size, num_pages=16384,
                         seed=1900 + 11 * T + page_size, poison_tail=True, extra_table_cols=2, **SHAPES[shape])
        assert mfma_kernel_selected(p)
        check_problem(p, impl=TUNED, num_splits=splits, what=f"{shape} page {page_size} T={T} splits={splits}")


@pytest.mark.parametrize("splits", [1, 3, 50])
@pytest.mark.parametrize("shape", list(SHAPES))
def test_key_ranges_do_not_change_the_result(shape, splits):
    p = make_problem(f"flex_sp_{shape}", seq_lens=[1000, 129, 64, 5, 3000], T=2, num_pages=2048, seed=1200 + splits,
                     poison_tail=True, **SHAPES[shape])
    check_problem(p, impl=TUNED, num_splits=splits, what=f"{shape} splits={splits}")


@pytest.mark.parametrize("shape", list(SHAPES))
def test_few_keys_and_peaky_rows(shape):
    """Short sequences with every key visible and strongly scaled queries: the
    weights go into the value product with 16 significant bits."""
    for seed, lens, gain in ((711, [2] * 30 + [3] * 10 + [1, 4, 5], 1.0), (1301, [900, 77, 2000], 8.0)):
        p = make_problem(f"flex_pk_{shape}", seq_lens=lens, T=2, num_pages=512, seed=seed, causal=0, q_gain=gain,
                         poison_tail=True, **SHAPES[shape])
        check_problem(p, impl=TUNED, what=f"{shape} seed {seed}")


@pytest.mark.parametrize("shape,T", [("gta64", 1), ("gta64", 2), ("gta96", 2), ("gqa128", 1)])
def test_repeat_calls_agree_bit_for_bit(shape, T):
    """Many short chunks with several sequences each (every chunk starts and ends
    inside a sequence, residual passes on most tiles): the result must not depend
    on timing.  The same call twenty times, every result equal to the first one
    and within tolerance of the oracle."""
    from gpu_util import run_gpu, compare
    p = make_problem(f"flex_rep_{shape}", seq_lens=LENS, T=T, page_size=64, num_pages=4096, seed=1707, poison_tail=True,
                     extra_table_cols=1, **SHAPES[shape])
    dp = DeviceProblem(p, poison_unused=True)
    ref_out, ref_lse = oracle.decode_problem(p)
    first = None
    for rep in range(20):
        out, lse = run_gpu(p, dp=dp, out_dtype=torch.float32, impl=TUNED)
        if first is None:
            first = (out, lse)
            compare(out, lse, ref_out, ref_lse, what=f"{shape} T={T}", bf16_out_allowance=False)
        else:
            assert np.array_equal(out, first[0]) and np.array_equal(lse, first[1]), f"{shape} T={T}: call {rep} differs from the first"


@pytest.mark.parametrize("shape", ["gta64", "gqa128"])
def test_large_ragged_batch_on_sampled_rows(shape):
    """A ragged batch of the size class of the benchmark's GTA configuration
    (64 sequences of 1000 to 12000 tokens), the automatic choice of chunks."""
    lens = uniform_lengths(64, 1000, 12000, 77)
    p = make_problem(f"flex_big_{shape}", seq_lens=lens, T=1, num_pages=16384, seed=1400, poison_tail=True, **SHAPES[shape])
    rng = np.random.default_rng(5)
    sel = sorted({(int(rng.integers(p.B)), 0, int(rng.integers(p.h_q))) for _ in range(300)})
    check_problem(p, sel=sel, impl=TUNED, what=f"{shape} large batch")


@pytest.mark.parametrize("shape,T", [("gta64", 1), ("gta64", 4), ("gta96", 1), ("gqa64", 2), ("gla128", 1)])
def test_hundreds_of_short_and_empty_sequences(shape, T):
    """More sequences than one pass of the prefix sums covers (64), most of them
    shorter than a chunk, every fifth one empty: chunks that hold many whole
    sequences, sequences cut at every position, empty rows filled by the merge
    kernel.  Every row against the oracle."""
    lens = uniform_lengths(333, 1, 400, 91 + T)
    lens[::5] = 0
    lens[7], lens[150], lens[332] = 5000, 2500, 3100
    p = make_problem(f"flex_many_{shape}", seq_lens=lens, T=T, page_size=32, num_pages=8192, seed=1800 + T, poison_tail=True,
                     extra_table_cols=1, **SHAPES[shape])
    assert mfma_kernel_selected(p)
    check_problem(p, impl=TUNED, what=f"{shape} many sequences T={T}")


@pytest.mark.parametrize("case", range(30))
def test_seeded_random_shapes(case):
    """Seeded sweep over the shapes of this kernel with other head counts (one to
    sixteen rows per group and query position, one or two groups per wave, several
    row blocks per group), query lengths, page sizes, batch sizes beyond one pass
    of the prefix sums, length mixes with empty sequences, chunk lengths and masks."""
    rng = np.random.default_rng(9500 + case)
    kind, h_c, d_v, d_r = [("gta", 4, 64, 32), ("gta", 2, 64, 32), ("gta", 4, 96, 48), ("gla", 2, 128, 32),
                           ("gqa", 4, 128, 0), ("gqa", 8, 64, 0), ("gta", 3, 64, 32), ("gla", 1, 128, 32),
                           ("gta", 1, 96, 48), ("gqa", 1, 128, 0)][case % 10]
    g_q = int(rng.choice([1, 3, 6, 8, 12, 16]))
    T = int(rng.integers(1, 5))
    B = int(rng.choice([1, 2, 5, 17, 70, 130]))
    lens = [int(x) for x in rng.choice([0, 0, 1, 2, 31, 32, 33, 64, 65, 127, 300, 900], size=B)]
    lens[int(rng.integers(B))] = int(rng.integers(1, 4000))
    page = int(rng.choice([32, 64, 64, 16, 4, 1]))
    kw = dict(d_r=d_r) if kind != "gqa" else {}
    p = make_problem(f"flex_rand{case}", kind=kind, seq_lens=lens, T=T, h_q=h_c * g_q, h_c=h_c, d_v=d_v, page_size=page,
                     num_pages=max(8192, 2 * sum(-(-n // page) for n in lens) + 64), seed=9600 + case, causal=int(rng.integers(0, 2)), poison_tail=True,
                     extra_table_cols=int(rng.integers(0, 3)), **kw)
    assert mfma_kernel_selected(p)
    check_problem(p, impl=TUNED, num_splits=int(rng.choice([0, 0, 1, 2, 7, 40])),
                  what=f"case {case} {kind} h_c={h_c} g_q={g_q} d_v={d_v} T={T} B={B} page={page}")


@pytest.mark.parametrize("index", [6, 7, 8])
def test_full_size_configs_on_sampled_rows(index):
    """The configurations the benchmark times on this kernel, at full size
    (128 sequences of 4096 to 32768 tokens), automatic chunks; seeded samples of
    rows, which the oracle computes one by one."""
    p = config(index)
    assert mfma_kernel_selected(p)
    rng = np.random.default_rng(600 + index)
    sel = sorted({(int(rng.integers(p.B)), 0, int(rng.integers(p.h_q))) for _ in range(160)})
    check_problem(p, sel=sel, impl=TUNED, what=f"cfg{index}")


def test_gqa_strided_caches_and_argument_checks():
    p = make_problem("gqa_strided", kind="gqa", seq_lens=[300, 0, 77, 1200], T=2, h_q=32, h_c=4, d_v=128, seed=1500,
                     num_pages=256, poison_tail=True)
    dp = DeviceProblem(p, poison_unused=True)
    ref_out, ref_lse = oracle.decode_problem(p)
    # keys and values as slices of pools with one more head per page
    kpool = torch.full((p.num_pages, p.h_c + 1, p.page_size, p.d_n), float("nan"), dtype=torch.bfloat16, device="cuda")
    kpool[:, :p.h_c] = dp.key_cache
    vpool = torch.full((p.num_pages, p.h_c + 1, p.page_size, p.d_v), float("nan"), dtype=torch.bfloat16, device="cuda")
    vpool[:, 1:] = dp.state_cache
    out, lse = gla.gqa_decode(dp.q_nope, kpool[:, :p.h_c], vpool[:, 1:], dp.page_table, dp.seq_lens, p.scale,
                              impl=TUNED, out_dtype=torch.float32)
    torch.cuda.synchronize()
    from gpu_util import compare
    compare(out.double().cpu().numpy(), lse.double().cpu().numpy(), ref_out, ref_lse, what="gqa strided", bf16_out_allowance=False)
    # a RoPE dim is not part of this entry point
    bad = torch.zeros(p.B, p.T, p.h_q, 64, dtype=torch.bfloat16, device="cuda")
    prm = gla.make_params(dp.q_nope, bad, dp.state_cache, torch.zeros(p.num_pages, p.page_size, 64, dtype=torch.bfloat16, device="cuda"),
                          dp.page_table, dp.seq_lens, p.scale, out=torch.empty(p.B, p.T, p.h_q, p.d_v, dtype=torch.bfloat16, device="cuda"),
                          lse=torch.empty(p.B, p.T, p.h_q, dtype=torch.float32, device="cuda"), workspace=None)
    assert gla.gla_decode_select_impl(prm, 2) == gla.GLA_ERR_INVALID_ARG
