"""GPU parity: aride_actor_loss_grad (actor loss of eq. (1) and its logit gradient) against the
CPU oracle.

fp32 gradient: |g - o| <= 1e-4 * |o| + the per-element bound of _util.grad_bound: where the factor
coef + beta*(log p_v + H) cancels, what is left is p_v times the element's factors times (the
absolute errors the second sweep inherits from the first sweep's tok_logp and tok_ent, measured
here, plus 16 fp32 roundings of its own).  An element of probability p_v is thus held to an
absolute error of the order p_v * 1e-6 of the row's gradient scale, the token's own entry
included.
bf16 gradient: bit-identical to the fp32 result rounded to nearest even, hence within one bf16
ulp (2^-7 relative) of the oracle.
"""
import numpy as np
import pytest
import torch

from paper_2410_14803_amd import binding as b
from paper_2410_14803_amd import synth
from _util import assert_close, bits_of, grad_bound, host_threads, npf

pytestmark = pytest.mark.gpu
DEV = "cuda"


def first_pass(logits, tokens, A, V=None):
    R = logits.shape[0]; N = R // A
    ws = b.Workspace(0)
    o = dict(tok_logp=torch.empty(R, device=DEV), tok_ent=torch.empty(R, device=DEV),
             step_logp=torch.empty(N, device=DEV), step_ent=torch.empty(N, device=DEV))
    b.score_logits(logits, tokens, A, ws, V=V, **o)
    return o


def step_inputs(N, seed):
    g = torch.Generator(device=DEV); g.manual_seed(seed)
    rho = torch.exp(0.5 * torch.randn(N, generator=g, device=DEV))
    target = torch.rand(N, generator=g, device=DEV) * 2 - 1
    base = torch.rand(N, generator=g, device=DEV) * 2 - 1
    pen = (torch.rand(N, generator=g, device=DEV) < 0.3).float()
    return rho, target, base, pen


def check_grad(got32, got16, want, logits, tokens, V, rho, target, base, o_score, fp, A, beta, scale, tag):
    """got32 / got16 [R, V] against the oracle's `want`; o_score / fp: the oracle's and the device's first sweep."""
    coef = np.repeat(npf(rho).astype(np.float64) * (npf(target).astype(np.float64) - npf(base)), A)
    extra = grad_bound(bits_of(logits), npf(tokens), V, coef, beta, scale, o_score["tok_logp"], o_score["tok_ent"],
                       npf(fp["tok_logp"]), npf(fp["tok_ent"]))
    if got32 is not None:
        err = np.abs(got32 - want)
        bound = 1e-4 * np.abs(want) + extra
        assert np.all(err <= bound), f"{tag}: fp32 gradient off; worst ratio {np.max(err / bound):.3f}"
    err16 = np.abs(got16 - want)
    bound16 = 2.0 ** -7 * np.abs(want) + extra
    assert np.all(err16 <= bound16), f"{tag}: bf16 gradient beyond one ulp; worst ratio {np.max(err16 / bound16):.3f}"


@pytest.mark.parametrize("V,pad,beta", [(1, 0, 0.1), (7, 1, 0.0), (64, 0, 0.01), (513, 3, 0.5), (2051, 5, 0.01),
                                        (8190, 2, 0.02), (8200, 8, 0.02), (12287, 1, 0.01), (12288, 0, 0.01),
                                        (32128, 0, 0.01), (33001, 3, 0.01)])
def test_small_shapes(oracle, V, pad, beta):
    print(f"case V={V} pad={pad}", flush=True)
    N, A = 5, 4
    R = N * A
    stride = V + pad
    logits = synth.logits_bf16(R, stride, seed=700 + V, device=DEV, heavy_tail=(V % 2 == 1))
    tokens = synth.action_tokens(logits[:, :V].contiguous(), seed=800 + V)
    tokens[6] = -1
    fp = first_pass(logits, tokens, A, V=V)
    rho, target, base, pen = step_inputs(N, 900 + V)
    scale, lam = 1.0 / N, 0.25
    g32 = torch.full((R, stride), 7.0, device=DEV)
    g16 = torch.full((R, stride), 7.0, dtype=torch.bfloat16, device=DEV)
    loss = torch.zeros(1, device=DEV)
    b.actor_loss_grad(logits, tokens, A, fp["tok_logp"], fp["tok_ent"], fp["step_logp"], fp["step_ent"], rho,
                      target, base, beta, scale, penalty=pen, lambda_pen=lam, grad=g32, loss=loss, V=V)
    b.actor_loss_grad(logits, tokens, A, fp["tok_logp"], fp["tok_ent"], fp["step_logp"], fp["step_ent"], rho,
                      target, base, beta, scale, grad=g16, V=V)
    torch.cuda.synchronize()
    o_loss, o_grad = oracle.actor_loss_grad(bits_of(logits), npf(tokens), A, npf(rho), npf(target), npf(base),
                                            beta, scale, penalty=npf(pen), lambda_pen=lam, V=V)
    o_score = oracle.score_logits(bits_of(logits), npf(tokens), A, V=V)
    check_grad(npf(g32)[:, :V].astype(np.float64), npf(g16.float())[:, :V].astype(np.float64), o_grad, logits, tokens,
               V, rho, target, base, o_score, fp, A, beta, scale, f"V={V}")
    assert_close(npf(loss), [o_loss], 1.0, "loss")
    # rounding the fp32 gradient to bf16 gives the bf16 gradient, bit for bit
    assert torch.equal(g32[:, :V].to(torch.bfloat16), g16[:, :V])
    assert torch.all(g32[6, :V] == 0)                 # padding row
    if pad:
        assert torch.all(g32[:, V:] == 7.0) and torch.all(g16[:, V:].float() == 7.0)   # columns >= V untouched


def test_masked_vocabulary_and_loss_only(oracle):
    V, A = 900, 2
    x = torch.randn(4, V, device=DEV) * 2
    x[0, ::2] = float("-inf")
    x[2, 5:] = -3.0e38
    logits = x.to(torch.bfloat16)
    tokens = torch.tensor([1, 3, 2, 7], dtype=torch.int32, device=DEV)
    fp = first_pass(logits, tokens, A)
    rho, target, base, pen = step_inputs(2, 5)
    g32 = torch.empty((4, V), device=DEV)
    loss = torch.zeros(1, device=DEV)
    b.actor_loss_grad(logits, tokens, A, fp["tok_logp"], fp["tok_ent"], fp["step_logp"], fp["step_ent"], rho,
                      target, base, 0.05, 0.5, grad=g32)
    b.actor_loss_grad(logits, tokens, A, None, None, fp["step_logp"], fp["step_ent"], rho, target, base,
                      0.05, 0.5, loss=loss)          # loss only: no logits needed
    torch.cuda.synchronize()
    o_loss, o_grad = oracle.actor_loss_grad(bits_of(logits), npf(tokens), A, npf(rho), npf(target), npf(base),
                                            0.05, 0.5)
    assert np.all(np.isfinite(npf(g32)))
    assert np.all(npf(g32)[0, ::2] == 0)             # masked vocabulary entries get no gradient
    o_score = oracle.score_logits(bits_of(logits), npf(tokens), A)
    check_grad(npf(g32).astype(np.float64), npf(g32.to(torch.bfloat16).float()).astype(np.float64), o_grad, logits,
               tokens, V, rho, target, base, o_score, fp, A, 0.05, 0.5, "masked")
    assert_close(npf(loss), [o_loss], 1.0, "loss-only")


def test_config1_full_size_sampled(oracle):
    cfg = synth.CONFIGS[1]
    seed = synth.BASE_SEED + cfg.index
    off = synth.trajectory_offsets(cfg, seed)
    N = int(off[-1]); R = N * cfg.A
    print(f"config1 actor R={R}", flush=True)
    logits = synth.logits_bf16(R, cfg.V, seed + 1, DEV)
    tokens = synth.action_tokens(logits, seed + 2)
    fp = first_pass(logits, tokens, cfg.A)
    rho, target, base, pen = step_inputs(N, 77)
    beta, scale = 0.01, 1.0 / N
    g16 = torch.empty((R, cfg.V), dtype=torch.bfloat16, device=DEV)
    loss = torch.zeros(1, device=DEV)
    b.actor_loss_grad(logits, tokens, cfg.A, fp["tok_logp"], fp["tok_ent"], fp["step_logp"], fp["step_ent"], rho,
                      target, base, beta, scale, penalty=pen, lambda_pen=0.1, grad=g16, loss=loss)
    torch.cuda.synchronize()
    g = np.random.default_rng(3)
    rows = np.unique(np.concatenate([[0, R - 1], g.integers(0, R, 2000)]))
    rt = torch.as_tensor(rows, device=DEV)
    steps = rows // cfg.A
    _, o_grad = oracle.actor_loss_grad(bits_of(logits[rt]), npf(tokens)[rows], 1, npf(rho)[steps], npf(target)[steps],
                                       npf(base)[steps], beta, scale)
    o_score = oracle.score_logits(bits_of(logits[rt]), npf(tokens)[rows], 1, nthreads=8)
    got16 = npf(g16[rt].float()).astype(np.float64)
    coef = np.abs(npf(rho)[steps].astype(np.float64) * (npf(target)[steps].astype(np.float64) - npf(base)[steps]))
    fp_rows = dict(tok_logp=fp["tok_logp"][rt], tok_ent=fp["tok_ent"][rt])
    check_grad(None, got16, o_grad, logits[rt], tokens[rt], cfg.V, torch.as_tensor(npf(rho)[steps]),
               torch.as_tensor(npf(target)[steps]), torch.as_tensor(npf(base)[steps]), o_score, fp_rows, 1, beta, scale,
               "config1 sampled rows")
    # the loss needs only per-step quantities: check it against the oracle's formula on the device's sums
    coef_all = npf(rho).astype(np.float64) * (npf(target).astype(np.float64) - npf(base))
    want = scale * np.sum(-coef_all * npf(fp["step_logp"]) - beta * npf(fp["step_ent"]) + 0.1 * npf(pen))
    assert_close(npf(loss), [want], 1.0, "loss at full size")
    # softmax is shift invariant: every gradient row sums to ~0 (bf16 rounding noise only)
    sums = g16[rt].float().sum(1).abs().cpu().numpy()
    assert np.all(sums <= 64 * 2.0 ** -8 * scale * (coef + beta * 12) + 1e-12)


def test_config1_full_size_every_row(oracle):
    # every element of the bf16 gradient of the learner batch (82 144 rows x 32 128) against the
    # oracle: rows go to the host once, the oracle and the comparison run over blocks of rows on
    # all host threads (the oracle's routine is called per block with A = 1 and per-row factors)
    from concurrent.futures import ThreadPoolExecutor
    cfg = synth.CONFIGS[1]
    seed = synth.BASE_SEED + cfg.index
    off = synth.trajectory_offsets(cfg, seed)
    N = int(off[-1]); R = N * cfg.A; V = cfg.V
    print(f"config1 actor, every row: R={R}", flush=True)
    logits = synth.logits_bf16(R, V, seed + 1, DEV)
    tokens = synth.action_tokens(logits, seed + 2)
    fp = first_pass(logits, tokens, cfg.A)
    rho, target, base, _ = step_inputs(N, 78)
    beta, scale = 0.01, 1.0 / N
    g16 = torch.empty((R, V), dtype=torch.bfloat16, device=DEV)
    b.actor_loss_grad(logits, tokens, cfg.A, fp["tok_logp"], fp["tok_ent"], fp["step_logp"], fp["step_ent"], rho,
                      target, base, beta, scale, grad=g16)
    torch.cuda.synchronize()
    bits = bits_of(logits)
    gbits = bits_of(g16)
    del logits, g16
    tok = npf(tokens)
    rows_of = lambda t: np.repeat(npf(t).astype(np.float64), cfg.A)
    rho_r, target_r, base_r = rows_of(rho), rows_of(target), rows_of(base)
    g_logp, g_ent = npf(fp["tok_logp"]), npf(fp["tok_ent"])
    o_score = oracle.score_logits(bits, tok, 1, nthreads=host_threads())
    print("first sweep compared, gradient blocks next", flush=True)
    assert_close(g_logp, o_score["tok_logp"], float(np.log(V)), "tok_logp")

    def block(r0):
        r1 = min(R, r0 + 512)
        sl = slice(r0, r1)
        _, want = oracle.actor_loss_grad(bits[sl], tok[sl], 1, rho_r[sl], target_r[sl], base_r[sl], beta, scale)
        got = (gbits[sl].astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
        extra = grad_bound(bits[sl], tok[sl], V, rho_r[sl] * (target_r[sl] - base_r[sl]), beta, scale,
                           o_score["tok_logp"][sl], o_score["tok_ent"][sl], g_logp[sl], g_ent[sl])
        bound = 2.0 ** -7 * np.abs(want) + extra
        err = np.abs(got - want)
        bad = int(np.count_nonzero(~(err <= bound)))
        return bad, float(np.max(err / bound))

    with ThreadPoolExecutor(max_workers=host_threads()) as pool:
        results = list(pool.map(block, range(0, R, 512)))
    bad = sum(r[0] for r in results)
    worst = max(r[1] for r in results)
    print(f"worst ratio to the bound {worst:.3f}", flush=True)
    assert bad == 0, f"{bad} gradient elements beyond one bf16 ulp plus the inherited bound; worst ratio {worst:.3f}"


def test_more_rows_than_one_launch_covers():
    # two-logit rows take one wave each and a launch covers 2^25 of them: 2^25 + 4 rows take two.
    # Uniform rows, rho * A = 1, scale 1: the gradient is -1/2 at the token and +1/2 beside it.
    R, V, A = (1 << 25) + 4, 2, 4
    N = R // A
    print(f"case actor R={R} V={V}", flush=True)
    logits = torch.zeros((R, V), dtype=torch.bfloat16, device=DEV)
    tokens = torch.zeros(R, dtype=torch.int32, device=DEV)
    tokens[-1] = 1
    fp = first_pass(logits, tokens, A)
    one, zero = torch.ones(N, device=DEV), torch.zeros(N, device=DEV)
    g32 = torch.full((R, V), float("nan"), device=DEV)
    b.actor_loss_grad(logits, tokens, A, fp["tok_logp"], fp["tok_ent"], fp["step_logp"], fp["step_ent"], one, one, zero,
                      0.01, 1.0, grad=g32)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(g32).any()), "a row was not written"
    body = g32[:-1]
    assert float((body[:, 0] + 0.5).abs().max()) < 1e-6 and float((body[:, 1] - 0.5).abs().max()) < 1e-6
    assert abs(float(g32[-1, 1]) + 0.5) < 1e-6 and abs(float(g32[-1, 0]) - 0.5) < 1e-6


def test_longest_row():
    # V = 2^31 - 1 logits in a row, the most a call accepts: element numbers up to the 32-bit limit.
    # A uniform row with rho * A = 1 and scale 1: every gradient element is 1/V but the token's,
    # which is 1/V - 1 (the entropy term vanishes: log p + H = 0).
    V = (1 << 31) - 1
    stride = 1 << 31
    torch.cuda.empty_cache()
    if torch.cuda.mem_get_info()[0] < (24 << 30):
        pytest.skip("needs 10 GB of free device memory")
    print(f"case actor V={V}", flush=True)
    logits = torch.zeros((1, stride), dtype=torch.bfloat16, device=DEV)
    tokens = torch.tensor([V - 1], dtype=torch.int32, device=DEV)
    fp = first_pass(logits, tokens, 1, V=V)
    one, zero = torch.ones(1, device=DEV), torch.zeros(1, device=DEV)
    g16 = torch.full((1, stride), 7.0, dtype=torch.bfloat16, device=DEV)
    b.actor_loss_grad(logits, tokens, 1, fp["tok_logp"], fp["tok_ent"], fp["step_logp"], fp["step_ent"], one, one, zero,
                      0.01, 1.0, grad=g16, V=V)
    torch.cuda.synchronize()
    body = g16[0, : V - 1].float()
    assert float(body.min()) == float(body.max())
    assert abs(float(body[0]) * V - 1.0) < 2.0 ** -7 + 1e-3          # one bf16 ulp, and the first sweep's log Z
    assert abs(float(g16[0, V - 1]) + 1.0) < 2.0 ** -7
    assert float(g16[0, V]) == 7.0                                    # the column past the row is untouched
