"""GPU parity: aride_score_logits (through the C ABI) against the CPU oracle."""
import math

import numpy as np
import pytest
import torch

from paper_2410_14803_amd import binding as b
from paper_2410_14803_amd import synth
from _util import assert_close, bits_of, ent_floor, npf, scored_config

pytestmark = pytest.mark.gpu
DEV = "cuda"


def run_gpu(logits, tokens, A, V=None):
    R = logits.shape[0]
    ws = b.Workspace(0)
    out = {k: torch.full((R,), 7.0, device=DEV) for k in ("tok_logp", "tok_ent")}
    out.update({k: torch.full((R // A,), 7.0, device=DEV) for k in ("step_logp", "step_ent")})
    b.score_logits(logits, tokens, A, ws, V=V, **out)
    torch.cuda.synchronize()
    st, _ = ws.status()
    return {k: npf(v) for k, v in out.items()}, st.flags


def compare(got, want, V, A, tag):
    assert_close(got["tok_logp"], want["tok_logp"], 1.0, f"{tag} tok_logp")
    assert_close(got["tok_ent"], want["tok_ent"], ent_floor(V), f"{tag} tok_ent")
    assert_close(got["step_logp"], want["step_logp"], 1.0, f"{tag} step_logp")
    assert_close(got["step_ent"], want["step_ent"], ent_floor(V), f"{tag} step_ent")


@pytest.mark.parametrize("V,stride_pad", [(1, 0), (7, 0), (8, 0), (63, 1), (64, 0), (513, 3), (2051, 5),
                                          (4096, 0), (8200, 8), (32128, 0), (40001, 1)])
def test_small_shapes_tiles_and_ragged_tails(oracle, V, stride_pad):
    # several vector tiles plus head/tail remainders; odd strides put rows off 16-byte alignment
    print(f"case V={V} pad={stride_pad}", flush=True)
    N, A = 6, 4
    R = N * A
    stride = V + stride_pad
    full = synth.logits_bf16(R, stride, seed=100 + V, device=DEV, heavy_tail=(V % 2 == 1))
    tokens = synth.action_tokens(full[:, :V].contiguous(), seed=200 + V)
    tokens[5] = -1
    got, flags = run_gpu(full, tokens, A, V=V)
    want = oracle.score_logits(bits_of(full), npf(tokens), A, V=V)
    compare(got, want, max(V, 2), A, f"V={V}")
    assert flags == 0
    assert got["tok_logp"][5] == 0 and got["tok_ent"][5] == 0


def test_uniform_logits_give_log_v():
    # closed form, no oracle involved: logp = -log V, H = log V
    for V in (32128, 151936, 1000):
        logits = torch.full((8, V), 1.5, dtype=torch.bfloat16, device=DEV)
        tokens = torch.arange(8, dtype=torch.int32, device=DEV)
        got, _ = run_gpu(logits, tokens, 2)
        assert_close(got["tok_logp"], np.full(8, -math.log(V)), 1.0, "uniform logp")
        assert_close(got["tok_ent"], np.full(8, math.log(V)), ent_floor(V), "uniform ent")


def test_bad_token_sets_flag_and_masks(oracle):
    V = 500
    logits = synth.logits_bf16(8, V, seed=7, device=DEV)
    tokens = torch.tensor([0, 1, V, 3, -5, 499, 500, 2], dtype=torch.int32, device=DEV)
    got, flags = run_gpu(logits, tokens, 4)
    want = oracle.score_logits(bits_of(logits), npf(tokens), 4)
    compare(got, want, V, 4, "bad-token")
    assert flags & b.ST_BAD_TOKEN
    assert got["tok_logp"][2] == 0 and got["tok_logp"][6] == 0


def test_masked_vocabulary_entries_and_extremes(oracle):
    # -inf logits (masked vocabulary), a dominant logit, and large offsets
    V = 3000
    x = torch.randn(6, V, device=DEV) * 2
    x[0, ::3] = float("-inf")
    x[1, 17] = 60.0
    x[2] += 200.0
    x[3] -= 300.0
    x[4, :2990] = float("-inf")
    x[5, 5:] = -3.0e38
    logits = x.to(torch.bfloat16)
    tokens = torch.tensor([1, 17, 5, 9, 2995, 2], dtype=torch.int32, device=DEV)
    got, flags = run_gpu(logits, tokens, 1)
    want = oracle.score_logits(bits_of(logits), npf(tokens), 1)
    compare(got, want, V, 1, "extremes")
    assert np.all(np.isfinite(got["tok_ent"]))


def test_adversarial_ordering_forces_rebase(oracle):
    # ascending rows make every group exceed the running reference; descending rows never do
    V = 20000
    base = torch.linspace(-40, 40, V, device=DEV)
    logits = torch.stack([base, base.flip(0), base * 0.1, -base.abs()]).to(torch.bfloat16)
    tokens = torch.tensor([V - 1, 0, 7, V // 2], dtype=torch.int32, device=DEV)
    got, _ = run_gpu(logits, tokens, 1)
    want = oracle.score_logits(bits_of(logits), npf(tokens), 1)
    compare(got, want, V, 1, "ordering")


def test_config0_full(oracle):
    cfg = synth.CONFIGS[0]
    seed = synth.BASE_SEED + cfg.index
    off = synth.trajectory_offsets(cfg, seed)
    R = int(off[-1]) * cfg.A
    logits = synth.logits_bf16(R, cfg.V, seed + 1, DEV)
    tokens = synth.action_tokens(logits, seed + 2)
    got, flags = run_gpu(logits, tokens, cfg.A)
    want = oracle.score_logits(bits_of(logits), npf(tokens), cfg.A, nthreads=8)
    compare(got, want, cfg.V, cfg.A, "config0")
    assert flags == 0


@pytest.mark.parametrize("ci", [1, 2])
def test_config_full_size_every_row(ci):
    # the learner batch (82 144 rows, 5.3 GB) and the large-vocabulary batch (131 072 rows of 304 KB,
    # 39.8 GB): every row and every step against the oracle, which reads the logits in 1 GB chunks
    case = scored_config(ci)
    cfg, got = case["cfg"], {k: npf(v) for k, v in case["got"].items()}
    assert case["flags"] == 0
    compare(got, case["want"], cfg.V, cfg.A, f"config{ci}")


def test_long_actions(oracle):
    # A larger than a wave: lanes stride over the step's rows
    N, A, V = 3, 300, 257
    logits = synth.logits_bf16(N * A, V, seed=31, device=DEV)
    tokens = synth.action_tokens(logits, seed=32)
    got, flags = run_gpu(logits, tokens, A)
    want = oracle.score_logits(bits_of(logits), npf(tokens), A)
    compare(got, want, V, A, "A=300")
    assert flags == 0


def test_step_sum_is_the_rounded_exact_sum_of_the_per_token_values():
    # fp64 accumulation of at most a few hundred fp32 values is exact to well below an fp32 ulp
    N, A, V = 64, 64, 4000
    logits = synth.logits_bf16(N * A, V, seed=35, device=DEV, heavy_tail=True)
    tokens = synth.action_tokens(logits, seed=36)
    got, _ = run_gpu(logits, tokens, A)
    exact_lp = got["tok_logp"].astype(np.float64).reshape(N, A).sum(1).astype(np.float32)
    exact_en = got["tok_ent"].astype(np.float64).reshape(N, A).sum(1).astype(np.float32)
    np.testing.assert_array_equal(got["step_logp"], exact_lp)
    np.testing.assert_array_equal(got["step_ent"], exact_en)


def test_nonfinite_values_propagate():
    V, A = 600, 4
    x = torch.randn(8, V, device=DEV)
    x[1, 5] = float("-inf")      # the chosen token is a masked vocabulary entry
    x[6, 9] = float("nan")       # a NaN logit poisons its row
    logits = x.to(torch.bfloat16)
    tokens = torch.tensor([0, 5, 2, 3, 4, 5, 6, 7], dtype=torch.int32, device=DEV)
    got, flags = run_gpu(logits, tokens, A)
    assert got["tok_logp"][1] == -np.inf and np.isnan(got["tok_logp"][6])
    assert got["step_logp"][0] == -np.inf and np.isnan(got["step_logp"][1])
    assert np.isfinite(got["tok_ent"][1]) and np.isnan(got["step_ent"][1])


@pytest.mark.parametrize("offset", [-20480.0, -512.0, 768.0, 24576.0])
def test_accuracy_does_not_depend_on_the_logits_magnitude(oracle, offset):
    # softmax is shift invariant; differences of bf16 values are exact in fp32, so a common
    # offset of any size must not cost accuracy (values are kept exactly representable in bf16)
    V, A = 5000, 2
    g = torch.Generator(device=DEV); g.manual_seed(3)
    step = 2.0 ** (int(np.floor(np.log2(abs(offset)))) - 7)           # bf16 spacing in offset's binade
    x = torch.randint(-30, 31, (8, V), generator=g, device=DEV).float() * step + offset   # stays below the next binade
    logits = x.to(torch.bfloat16)
    assert torch.equal(logits.float(), x)
    tokens = synth.action_tokens(logits, seed=4)
    got, _ = run_gpu(logits, tokens, A)
    want = oracle.score_logits(bits_of(logits), npf(tokens), A)
    compare(got, want, V, A, f"offset {offset}")


@pytest.mark.parametrize("V", [500, 32128, 151936])      # one wave per row, 8 and 16 waves per row
def test_timed_entry_point_gives_the_same_results_and_a_kernel_time(V):
    import time
    cfg = synth.CONFIGS[0]
    R, A = 2560 if V < 100000 else 512, cfg.A
    logits = synth.logits_bf16(R, V, seed=77, device=DEV)
    tokens = synth.action_tokens(logits, seed=78)
    ws = b.Workspace(0)
    f = lambda n: torch.full((n,), 7.0, device=DEV)
    plain = [f(R), f(R), f(R // A), f(R // A)]
    timed = [f(R), f(R), f(R // A), f(R // A)]
    b.score_logits(logits, tokens, A, ws, *plain)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(); e1.record()                       # creates the HIP events
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    b.score_logits(logits, tokens, A, ws, *timed, sweep_events=(e0, e1))
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    for p, t in zip(plain, timed):
        assert torch.equal(p, t)
    ms = e0.elapsed_time(e1)
    # no faster than twice the HBM peak rate (a batch this small may sit in the last-level cache)
    assert R * V * 2 / 16e12 * 1e3 < ms <= wall_ms, (ms, wall_ms)
    # both events are required
    with pytest.raises(b.ArideError) as err:
        b._check("aride_score_logits_timed", b.lib().aride_score_logits_timed(
            b._p(logits), R, V, V, b._p(tokens), A, None, None, None, None, ws.ptr, ws.nbytes, None, None, None))
    assert err.value.rc == b.E_NULL


@pytest.mark.parametrize("V,stride_pad", [(8192, 0), (8193, 3), (8199, 1), (12345, 5), (16384 + 511, 2), (65536, 0),
                                          (151936, 0), (200001, 7)])
def test_several_waves_per_row_path(oracle, V, stride_pad):
    # long rows: each is shared by the 4, 8 or 16 waves of a workgroup
    print(f"case V={V} pad={stride_pad}", flush=True)
    N, A = 5, 3
    R = N * A
    stride = V + stride_pad
    full = synth.logits_bf16(R, stride, seed=900 + V, device=DEV, heavy_tail=True)
    q = V // 4
    full[1, :q] = float("-inf")                      # a whole quarter masked out
    full[2, q:2 * q] = float("-inf")
    full[3, 3 * q:V] = -3.0e38                       # ... or hugely negative
    for r, col in ((4, 5), (5, q + 77), (6, 2 * q + 1), (7, V - 1)):
        full[r, col] = 60.0                          # a dominant logit in each quarter in turn
    tokens = synth.action_tokens(full[:, :V].float().clamp(min=-1e30).to(torch.bfloat16).contiguous(), seed=901 + V)
    tokens[4], tokens[5], tokens[6], tokens[7] = 5, q + 77, 2 * q + 1, 0
    tokens[8] = -1
    tokens[9] = V                                     # out of range: masked, flagged
    got, flags = run_gpu(full, tokens, A, V=V)
    tok_o = npf(tokens).copy()
    tok_o[9] = -1
    want = oracle.score_logits(bits_of(full), tok_o, A, V=V)
    compare(got, want, V, A, f"split V={V}")
    assert flags == b.ST_BAD_TOKEN
    assert got["tok_logp"][8] == 0 and got["tok_ent"][8] == 0 and got["tok_logp"][9] == 0


@pytest.mark.parametrize("V", [8184, 8192, 24568, 24576, 98296, 98304, 98304 + 8 * 16 * 64 + 3])
def test_row_lengths_where_the_number_of_waves_per_row_changes(oracle, V):
    # rows below 16 KB take one wave each; from 1024, 3072 and 12288 16-byte vectors on a row is
    # shared by 4, 8 and 16 waves
    print(f"case V={V}", flush=True)
    R, A = 10, 2
    logits = synth.logits_bf16(R, V + 3, seed=950 + V, device=DEV, heavy_tail=True)
    tokens = synth.action_tokens(logits[:, :V].contiguous(), seed=951 + V)
    tokens[3] = -1
    got, flags = run_gpu(logits, tokens, A, V=V)
    want = oracle.score_logits(bits_of(logits), npf(tokens), A, V=V, nthreads=8)
    compare(got, want, V, A, f"V={V}")
    assert flags == 0


def test_more_rows_than_32_bits_count():
    # R = 2^31 + 4096 rows of two logits: row numbers and row offsets beyond 32 bits.  Equal logits
    # make every row uniform: log p = -ln 2, H = ln 2.
    R, V = (1 << 31) + 4096, 2
    torch.cuda.empty_cache()
    if torch.cuda.mem_get_info()[0] < (60 << 30):
        pytest.skip("needs 40 GB of free device memory")
    print(f"case R={R} V={V}", flush=True)
    logits = torch.zeros((R, V), dtype=torch.bfloat16, device=DEV)
    logits[-1, 1] = 3.0                                # the last row is not uniform: it must be reached, and only it
    tokens = torch.zeros(R, dtype=torch.int32, device=DEV)
    ws = b.Workspace(0)
    lp = torch.full((R,), float("nan"), device=DEV)
    en = torch.full((R,), float("nan"), device=DEV)
    b.score_logits(logits, tokens, 128, ws, tok_logp=lp, tok_ent=en)      # 2^24 + 32 steps of 128 tokens
    torch.cuda.synchronize()
    st, rc = ws.status()
    assert rc == b.OK and st.flags == 0
    ln2 = float(np.log(2.0))
    body_lp, body_en = lp[:-1], en[:-1]
    assert float(body_lp.min()) == float(body_lp.max()) and abs(float(body_lp[0]) + ln2) < 1e-6
    assert float(body_en.min()) == float(body_en.max()) and abs(float(body_en[0]) - ln2) < 1e-6
    z = np.log(1.0 + np.exp(3.0))
    p1 = np.exp(3.0 - z)
    assert abs(float(lp[-1]) - (0.0 - z)) < 1e-5
    assert abs(float(en[-1]) - (-(1 - p1) * np.log(1 - p1) - p1 * np.log(p1))) < 1e-5


def test_more_rows_than_one_launch_covers_with_several_waves_per_row():
    # 8192-logit rows are shared by 4 waves: a launch covers 2^23 of them; 2^23 + 24 rows take two.
    # Uniform rows: log p = -ln V, H = ln V; the last row carries one larger logit.
    R, V = (1 << 23) + 24, 8192
    torch.cuda.empty_cache()
    if torch.cuda.mem_get_info()[0] < (180 << 30):
        pytest.skip("needs 140 GB of free device memory")
    print(f"case R={R} V={V}", flush=True)
    logits = torch.zeros((R, V), dtype=torch.bfloat16, device=DEV)
    logits[-1, 5] = 4.0
    tokens = torch.zeros(R, dtype=torch.int32, device=DEV)
    ws = b.Workspace(0)
    lp = torch.full((R,), float("nan"), device=DEV)
    en = torch.full((R,), float("nan"), device=DEV)
    b.score_logits(logits, tokens, 8, ws, tok_logp=lp, tok_ent=en)
    torch.cuda.synchronize()
    lnv = float(np.log(V))
    assert float(lp[:-1].min()) == float(lp[:-1].max()) and abs(float(lp[0]) + lnv) < 1e-5
    assert float(en[:-1].min()) == float(en[:-1].max()) and abs(float(en[0]) - lnv) < 1e-5
    z = np.log(V - 1 + np.exp(4.0))
    assert abs(float(lp[-1]) + z) < 1e-5


def test_longest_row():
    # V = 2^31 - 1 logits in a row, the most a call accepts (two rows): element numbers inside a row
    # run up to the 32-bit limit.  Uniform rows: log p = -ln V, H = ln V; the second row has one
    # logit 20 above the rest at the very end, and that is its token.
    V = (1 << 31) - 1
    stride = 1 << 31
    torch.cuda.empty_cache()
    if torch.cuda.mem_get_info()[0] < (20 << 30):
        pytest.skip("needs 9 GB of free device memory")
    print(f"case V={V}", flush=True)
    logits = torch.zeros((2, stride), dtype=torch.bfloat16, device=DEV)
    logits[1, V - 1] = 20.0
    logits[:, V:] = 50.0                                  # beyond the row: must not be read
    tokens = torch.tensor([7, V - 1], dtype=torch.int32, device=DEV)
    ws = b.Workspace(0)
    lp = torch.full((2,), float("nan"), device=DEV)
    en = torch.full((2,), float("nan"), device=DEV)
    b.score_logits(logits, tokens, 1, ws, tok_logp=lp, tok_ent=en, V=V)
    torch.cuda.synchronize()
    st, rc = ws.status()
    assert rc == b.OK and st.flags == 0
    lnv = float(np.log(float(V)))
    assert abs(float(lp[0]) + lnv) < 1e-4 * lnv and abs(float(en[0]) - lnv) < 1e-4 * lnv
    z = np.log(float(V - 1) + np.exp(20.0))
    p1 = np.exp(20.0 - z)
    h = -(V - 1) * np.exp(-z) * (-z) - p1 * np.log(p1)
    assert abs(float(lp[1]) - (20.0 - z)) < 1e-4 * abs(20.0 - z) + 1e-6
    assert abs(float(en[1]) - h) < 1e-4 * h


def test_most_steps_and_longest_step():
    # R / A = 2^25 - 1 steps of one token (the most the per-step sums accept), and two steps of 2^20
    # tokens each: per-step values are the sums of the per-token ones
    for R, A in (((1 << 25) - 1, 1), (1 << 21, 1 << 20)):
        print(f"case R={R} A={A}", flush=True)
        V = 2
        logits = torch.zeros((R, V), dtype=torch.bfloat16, device=DEV)
        tokens = torch.zeros(R, dtype=torch.int32, device=DEV)
        ws = b.Workspace(0)
        N = R // A
        out = dict(tok_logp=torch.full((R,), float("nan"), device=DEV), tok_ent=torch.full((R,), float("nan"), device=DEV),
                   step_logp=torch.full((N,), float("nan"), device=DEV), step_ent=torch.full((N,), float("nan"), device=DEV))
        b.score_logits(logits, tokens, A, ws, **out)
        torch.cuda.synchronize()
        ln2 = float(np.log(2.0))
        for k, sign in (("step_logp", -1.0), ("step_ent", 1.0)):
            v = out[k]
            assert float(v.min()) == float(v.max()), k
            assert abs(float(v[0]) - sign * A * ln2) <= 1e-6 * A * ln2, k
