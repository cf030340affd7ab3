"""GPU parity of ef_token_dist (intra-batch diversity Dist(t), paper Sec. 2.2) against the CPU oracle.

Tolerance: the inputs are bf16, their products are exact in fp32, the inner products and squared
norms are fp32 sums over d terms (relative error about 1e-6 of n_i + n_j), the distance of a pair
at typical separation sqrt(n_i + n_j) therefore carries a relative error of about 1e-6, and the
per-token and total sums are taken in fp64.  Per-token values are compared to 1e-5 relative (plus
1e-5 absolute per earlier token), the total to 1e-6 relative.  Integer-valued inputs make every
fp32 sum exact; then only the correctly rounded fp32 square roots differ from fp64 (6e-8).
Batches of up to 256 tokens take a kernel that sums the squared differences directly in fp32 (the same
error model without the cancellation of n_i + n_j - 2 <v_i, v_j>); the tests below reach it through the
default form and the Gram kernels through the forced forms."""
import sys

import numpy as np
import pytest
import torch

from paper_2510_26730_amd import binding as ef
from paper_2510_26730_amd import synth

from helpers import dev_u16

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def make_ctx(d, max_tokens):
    return ef.ef_create(n_layers=1, d_model=d, n_experts=8, top_k=2, d_ff=64, d_ff_shared=0, slots_total=1,
                        slots_per_layer_max=0, max_tokens=max_tokens, h_max=1, renorm_topk=1, flags=0)


def run_dist(ctx, h, T, want_tokens=True):
    hd = dev_u16(h)
    tok = torch.full((T,), -1.0, dtype=torch.float32, device="cuda") if want_tokens else None
    tot = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    ef.ef_token_dist(ctx, hd, T, tok, tot, torch.cuda.current_stream())
    torch.cuda.synchronize()
    return (tok.cpu().numpy() if want_tokens else None), float(tot.cpu().numpy()[0])


@pytest.mark.parametrize("T,d", [(1, 64), (2, 64), (37, 64), (64, 512), (65, 192), (130, 192), (257, 256),
                                 (300, 128), (513, 64)])
def test_integer_tokens_match_oracle(oracle_mod, T, d):
    """Exact arithmetic case; every fourth token repeats an earlier one (distance exactly 0)."""
    say(f"dist integer tokens T={T} d={d}")
    rng = np.random.default_rng(1000 + T + d)
    v = rng.integers(-2, 3, size=(T, d)).astype(np.float32)
    for j in range(3, T, 4):
        v[j] = v[j // 2]
    h = synth.f32_to_bf16(v)
    ctx = make_ctx(d, max(T, 64))
    try:
        tok, tot = run_dist(ctx, h, T)
    finally:
        ef.ef_destroy(ctx)
    ref = oracle_mod.token_dist(h)
    np.testing.assert_allclose(tok, ref, rtol=1e-6, atol=1e-6)
    assert abs(tot - ref.sum()) <= 1e-6 * max(ref.sum(), 1.0)
    assert tok[0] == 0.0


@pytest.mark.parametrize("cfg_name,T", [("tiny", 64), ("tiny", 31), ("qwen15_moe", 640), ("deepseek_v2_lite", 1056)])
def test_gaussian_tokens_match_oracle(oracle_mod, cfg_name, T):
    cfg = synth.CONFIGS[cfg_name]
    say(f"dist gaussian tokens {cfg_name} T={T} d={cfg.d}")
    h = synth.hidden(cfg, 0, T)
    ctx = make_ctx(cfg.d, T)
    try:
        tok, tot = run_dist(ctx, h, T)
        tok2, tot2 = run_dist(ctx, h, T)
        _, tot3 = run_dist(ctx, h, T, want_tokens=False)
    finally:
        ef.ef_destroy(ctx)
    ref = oracle_mod.token_dist(h)
    np.testing.assert_allclose(tok, ref, rtol=1e-5, atol=1e-5 * T)
    assert abs(tot - ref.sum()) <= 1e-6 * ref.sum()
    assert np.array_equal(tok, tok2) and tot == tot2 == tot3, "not bit-reproducible"


def test_total_is_permutation_invariant(oracle_mod):
    cfg = synth.CONFIGS["tiny"]
    T = 200
    h = synth.hidden(cfg, 0, T)
    perm = np.random.default_rng(5).permutation(T)
    ctx = make_ctx(cfg.d, T)
    try:
        _, a = run_dist(ctx, h, T)
        _, b = run_dist(ctx, np.ascontiguousarray(h[perm]), T)
    finally:
        ef.ef_destroy(ctx)
    assert abs(a - b) <= 1e-6 * a
    assert abs(a - oracle_mod.token_dist(h).sum()) <= 1e-6 * a


def test_full_size_prefill_batch_sampled(oracle_mod):
    """T = 8192, d = 4096 (the prefill configuration): sampled tokens against the oracle, and the
    total against the fp64 sum of the per-token values (the oracle would need 4e11 operations)."""
    cfg = synth.CONFIGS["mixtral_prefill"]
    T = 8192
    say("dist full size: T=8192 d=4096")
    h = synth.hidden(cfg, 0, T)
    ctx = make_ctx(cfg.d, T)
    try:
        tok, tot = run_dist(ctx, h, T)
    finally:
        ef.ef_destroy(ctx)
    js = np.sort(np.random.default_rng(9).permutation(T)[:12]).astype(np.int32)
    js = np.concatenate([js, np.array([0, 1, 63, 64, 255, 256, T - 1], dtype=np.int32)])
    ref = oracle_mod.token_dist(h, js)
    np.testing.assert_allclose(tok[js], ref, rtol=1e-5, atol=1e-5 * T)
    assert abs(tot - tok.astype(np.float64).sum()) <= 1e-6 * tot
    assert np.all(np.isfinite(tok)) and np.all(tok[1:] > 0)


@pytest.mark.parametrize("T,d", [(1, 64), (33, 64), (257, 128), (300, 192), (1025, 64), (1400, 256), (2304, 64),
                                 (5900, 64)])
def test_both_gram_forms_give_the_same_bits_and_match_oracle(oracle_mod, T, d):
    """The Gram blocks staged through LDS (256 x 256, numbered in strips over the upper triangle) against the
    register-fed blocks and the oracle, at sizes of 1 to 9 block columns with ragged last blocks, and at 24 block
    columns (300 blocks: the 44 past the first round of 256 run as quarters)."""
    say(f"dist forms T={T} d={d}")
    rng = np.random.default_rng(4000 + T)
    h = synth.f32_to_bf16(rng.standard_normal((T, d)).astype(np.float32))
    ctx = make_ctx(d, max(T, 64))
    try:
        out = {}
        for form in (1, 2):
            ef.ef_set_tuning(ctx, dist_form=form)
            out[form] = run_dist(ctx, h, T)
    finally:
        ef.ef_destroy(ctx)
    assert np.array_equal(out[1][0], out[2][0]) and out[1][1] == out[2][1]
    ref = oracle_mod.token_dist(h)
    np.testing.assert_allclose(out[2][0], ref, rtol=1e-5, atol=1e-5 * T)
    assert abs(out[2][1] - ref.sum()) <= 1e-6 * max(ref.sum(), 1.0)


def test_argument_errors():
    ctx = make_ctx(64, 64)
    try:
        tot = torch.zeros(1, dtype=torch.float64, device="cuda")
        h = torch.zeros(64 * 64, dtype=torch.int16, device="cuda")
        for bad_T in (0, 65):
            with pytest.raises(ef.EfError) as e:
                ef.ef_token_dist(ctx, h, bad_T, None, tot, torch.cuda.current_stream())
            assert e.value.code == ef.EF_EINVAL
        with pytest.raises(ef.EfError):
            ef.ef_token_dist(ctx, None, 8, None, tot, torch.cuda.current_stream())
    finally:
        ef.ef_destroy(ctx)
