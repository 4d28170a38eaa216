"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Integer and byte results are bit-exact; floating-point results are within
|gpu - ref| <= 2e-3 + 1e-2 * |ref| (bf16 inputs, fp32 accumulation)."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2605_16360_amd import binding as pk
from paper_2605_16360_amd import synth

pytestmark = pytest.mark.gpu
ATOL, RTOL = 2e-3, 1e-2


def assert_close(gpu: torch.Tensor, ref: torch.Tensor, what: str):
    g, r = gpu.detach().double().cpu(), ref.double()
    assert g.shape == r.shape, (g.shape, r.shape)
    assert bool(torch.isfinite(g).all()), f"{what}: non-finite values"
    err = (g - r).abs()
    bound = ATOL + RTOL * r.abs()
    worst = int(torch.argmax(err - bound))
    assert bool((err <= bound).all()), (f"{what}: max abs err {float(err.max()):.3e}, worst at flat {worst}: "
                                        f"gpu {float(g.flatten()[worst])} ref {float(r.flatten()[worst])}")


def _ctx(case, weights=None):
    ctx = pk.proxykv_create(pk.config_for_case(case))
    if weights is not None:
        pk.proxykv_set_mapper_weights(ctx, weights)
    return ctx


# ----------------------------------------------------------------------------------------------
# top-k and compaction: bit-exact
# ----------------------------------------------------------------------------------------------

@pytest.mark.parametrize("N,K", [(1, 1), (17, 5), (1000, 300), (1024, 1024), (1025, 1), (5000, 1500), (32771, 9830),
                                 (70001, 21000)])
def test_topk_bit_exact(N, K):
    ctx = _ctx(synth.CASES["tiny"])
    g = torch.Generator().manual_seed(N + K)
    s = torch.randn(7, N, generator=g)
    s[1] = torch.round(s[1] * 4) / 4             # heavy ties
    s[2] = 0.5                                   # all equal
    s[3] = torch.round(s[3])
    if N > 8:
        s[4, ::5] = float("nan")
        s[5, 1], s[5, 2], s[5, 3], s[5, 4] = -0.0, 0.0, float("inf"), float("-inf")
        s[5, 5:] = torch.where(s[5, 5:].abs() < 0.5, torch.zeros(()), s[5, 5:])
        s[5, 7::2] *= -1.0                       # produces -0.0 next to +0.0
    s[6] = s[6] * 1e-3 + 0.25                    # narrow range: many shared high radix digits
    ref = oracle.topk(s, K)
    got = pk.proxykv_topk(ctx, s.cuda(), K)
    torch.cuda.synchronize()
    assert torch.equal(got.cpu(), ref)


@pytest.mark.parametrize("N", [36863, 36864, 36865, 40000, 45057, 90113, 170000])
def test_topk_bit_exact_around_the_kernel_switch(N):
    """Rows of up to 36 864 scores are selected by one workgroup, longer ones are split into parts of at most 45 056
    (one part, two parts, three parts with a ragged last one, four parts)."""
    ctx = _ctx(synth.CASES["tiny"])
    g = torch.Generator().manual_seed(N)
    s = torch.randn(5, N, generator=g)
    s[1] = torch.round(s[1] * 3) / 3
    s[2] = -7.5
    s[3, N // 2:] = s[3, :N - N // 2].clone()        # every value twice: the tie rule decides half of the cut
    for K in (1, N // 3, N - 1, N):
        got = pk.proxykv_topk(ctx, s.cuda(), K)
        torch.cuda.synchronize()
        assert torch.equal(got.cpu(), oracle.topk(s, K)), (N, K)


def test_compact_bit_exact():
    ctx = _ctx(synth.CASES["tiny"])
    g = torch.Generator().manual_seed(3)
    for (L, H, N, D, K) in [(2, 3, 700, 128, 211), (1, 2, 130, 64, 130), (1, 1, 9, 128, 1), (1, 2, 300, 256, 77), (2, 1, 257, 32, 100),
                            (1, 1, 100, 8, 33)]:
        kv = torch.randn(2, L, H, N, D, generator=g).to(torch.bfloat16)
        s = torch.randn(L * H, N, generator=g)
        idx = oracle.topk(s, K).view(L, H, K)
        k_out, v_out = pk.proxykv_compact(ctx, kv[0].cuda(), kv[1].cuda(), idx.cuda())
        torch.cuda.synchronize()
        assert torch.equal(k_out.cpu().view(torch.int16), oracle.compact(kv[0], idx).view(torch.int16))
        assert torch.equal(v_out.cpu().view(torch.int16), oracle.compact(kv[1], idx).view(torch.int16))


def test_compact_inplace_and_mask_bit_exact():
    """The cache as its own destination: tokens 0 .. K-1 equal the out-of-place gather, the rest is untouched;
    the byte mask marks exactly the kept tokens.  Dense kept sets (sources right behind destinations), K = N,
    K = 1, several chunks of 128 with a ragged last one, unaligned mask rows."""
    ctx = _ctx(synth.CASES["tiny"])
    g = torch.Generator().manual_seed(4)
    for (L, H, N, D, K) in [(2, 3, 700, 128, 211), (1, 2, 130, 64, 130), (1, 1, 9, 128, 1), (1, 2, 1000, 128, 999),
                            (2, 2, 1537, 128, 640), (1, 3, 333, 256, 129)]:
        kv = torch.randn(2, L, H, N, D, generator=g).to(torch.bfloat16)
        s = torch.randn(L * H, N, generator=g)
        idx = oracle.topk(s, K).view(L, H, K)
        k, v = kv[0].cuda(), kv[1].cuda()
        pk.proxykv_compact_inplace(ctx, k, v, idx.cuda())
        m = pk.proxykv_mask(ctx, idx.cuda(), N)
        torch.cuda.synchronize()
        for got, src in ((k, kv[0]), (v, kv[1])):
            assert torch.equal(got[..., :K, :].cpu().view(torch.int16), oracle.compact(src, idx).view(torch.int16)), (N, K)
            assert torch.equal(got[..., K:, :].cpu().view(torch.int16), src[..., K:, :].view(torch.int16)), (N, K)
        assert torch.equal(m.cpu(), oracle.mask(idx, N)), (N, K)


def test_pooled_budget_bit_exact():
    """One budget per layer shared by its heads: kept flat indices, per-head counts, and the ragged in-place
    compaction, against the oracle.  Covers short rows (register-resident selection) and long ones, heads that
    get nothing, a head that gets everything it has, ties across heads."""
    ctx = _ctx(synth.CASES["tiny"])
    g = torch.Generator().manual_seed(5)
    for (L, H, N, D, K) in [(2, 4, 700, 128, 211), (1, 3, 130, 64, 130), (1, 1, 9, 128, 1), (3, 8, 6000, 128, 1800),
                            (1, 2, 1537, 256, 300), (2, 5, 333, 64, 7)]:
        s = torch.randn(L, H, N, generator=g)
        s[0, 0] += 4.0                                  # head 0 of layer 0 takes as much as it can
        if H > 2:
            s[0, 2] -= 8.0                              # and head 2 gets nothing
        if L > 1:
            s[1] = torch.round(s[1] * 2) / 2            # ties across heads
        flat_ref, counts_ref = oracle.topk_pooled(s, K)
        flat, counts = pk.proxykv_topk_pooled(ctx, s.cuda(), K)
        torch.cuda.synchronize()
        assert torch.equal(flat.cpu(), flat_ref), (N, K)
        assert torch.equal(counts.cpu(), counts_ref), (N, K)
        kv = torch.randn(2, L, H, N, D, generator=g).to(torch.bfloat16)
        k, v = kv[0].cuda(), kv[1].cuda()
        pk.proxykv_compact_pooled(ctx, k, v, flat, counts)
        torch.cuda.synchronize()
        for l in range(L):
            start = 0
            for h in range(H):
                c = int(counts_ref[l, h])
                tok = (flat_ref[l, start:start + c].to(torch.int64) - h * N)
                start += c
                for got, src in ((k, kv[0]), (v, kv[1])):
                    assert torch.equal(got[l, h, :c].cpu().view(torch.int16), src[l, h][tok].view(torch.int16)), (N, K, l, h)
                    assert torch.equal(got[l, h, c:].cpu().view(torch.int16), src[l, h, c:].view(torch.int16)), (N, K, l, h)


def test_prune_selection_and_gather_in_one_launch_equals_two_launches():
    """proxykv_prune with the Top-K kernel gathering the kept tokens itself (the default) against the same call with the
    two kernels one after the other: same bits, for rows one workgroup selects and for rows split over several."""
    for (N, keep) in ((700, 0.3), (40000, 0.25)):
        case = synth.scaled_case(synth.CASES["llama_8k"], name=f"fused_{N}", L_s=1, H_q=2, H_kv=1, d=64, L_l=2, H_l=3, N=N, N_q=64,
                                 chunk=64, n_planted=2)
        q, kc, kr = synth.make_proxy_qk(case, device="cuda")
        k_t, v_t = synth.make_target_kv(case, device="cuda")
        ctx = _ctx(case, synth.make_mapper_weights(case.H_kv, case.H_l))
        outs = []
        for on in (True, False):
            pk.proxykv_set_fused_select(ctx, on)
            k_out, v_out, idx, K = pk.proxykv_prune(ctx, q, kc, kr, case.chunk, keep, k_t, v_t)
            torch.cuda.synchronize()
            outs.append((idx.clone(), k_out.view(torch.int16).clone(), v_out.view(torch.int16).clone()))
        for a, b in zip(*outs):
            assert torch.equal(a, b), N
        assert torch.equal(outs[0][1].cpu(), oracle.compact(k_t.cpu(), outs[0][0].cpu()).view(torch.int16))
        pk.proxykv_destroy(ctx)


# ----------------------------------------------------------------------------------------------
# scoring
# ----------------------------------------------------------------------------------------------

SCORE_CASES = {
    # several key/query tiles, ragged tails, chunk boundaries that cut query blocks
    "d64_ragged": dict(L_s=2, H_q=4, H_kv=2, d=64, N=1000, N_q=700, chunk=300, n_planted=6),
    "d64_gqa7": dict(L_s=1, H_q=14, H_kv=2, d=64, N=1500, N_q=1500, chunk=512, n_planted=8),
    "d128": dict(L_s=2, H_q=6, H_kv=2, d=128, N=900, N_q=640, chunk=256, n_planted=6),
    "one_query": dict(L_s=1, H_q=1, H_kv=1, d=64, N=5, N_q=1, chunk=1, n_planted=0),
    "small_chunks": dict(L_s=1, H_q=2, H_kv=1, d=64, N=300, N_q=300, chunk=17, n_planted=3),
}


def _score_case(name):
    return synth.scaled_case(synth.CASES["llama_8k"], name=name, L_l=1, H_l=2, **SCORE_CASES[name])


@pytest.mark.parametrize("name", list(SCORE_CASES))
def test_score_matches_oracle(name):
    case = _score_case(name)
    q, kc, kr = synth.make_proxy_qk(case)
    ref = oracle.score(q.double(), kc.double(), kr.double(), case.chunk)
    ctx = _ctx(case)
    x = pk.proxykv_score(ctx, q.cuda(), kc.cuda(), kr.cuda(), case.chunk)
    torch.cuda.synchronize()
    assert_close(x, ref, f"score[{name}]")
    x_min, x_max = float(x.min()), float(x.max())
    assert x_min >= 0.0 and x_max <= 1.0, (x_min, x_max)


@pytest.mark.parametrize("name", list(SCORE_CASES))
def test_score_sum_form_matches_oracle(name):
    """reduce = SUM: the accumulation over the query axis that Sec. 3 prints, over all heads of the group."""
    case = _score_case(name)
    q, kc, kr = synth.make_proxy_qk(case)
    ref = oracle.score(q.double(), kc.double(), kr.double(), case.chunk, reduce="sum")
    cfg = pk.config_for_case(case)
    cfg.reduce = pk.PROXYKV_REDUCE_SUM
    ctx = pk.proxykv_create(cfg)
    x = pk.proxykv_score(ctx, q.cuda(), kc.cuda(), kr.cuda(), case.chunk)
    torch.cuda.synchronize()
    assert_close(x, ref, f"score sum[{name}]")
    # every query row spends at most all of its probability on the context keys
    assert float(x.sum(dim=-1).max()) <= case.G * case.N_q * (1.0 + 1e-5)


@pytest.mark.parametrize("name", list(SCORE_CASES))
def test_score_self_matches_oracle(name):
    """The feature as Sec. 3 prints it: causal self-attention of the sequence, summed over queries and group heads."""
    case = _score_case(name)
    q, _, k = synth.make_proxy_qk(case)                 # the reconstruction keys serve as the sequence's own keys
    ref = oracle.score_self(q.double(), k.double())
    ctx = _ctx(case)
    x = pk.proxykv_score_self(ctx, q.cuda(), k.cuda())
    torch.cuda.synchronize()
    assert_close(x, ref, f"score_self[{name}]")
    # every query row is a probability vector over its visible keys
    total = x.double().sum(dim=-1).cpu()
    assert torch.allclose(total, torch.full_like(total, float(case.G * case.N_q)), rtol=1e-4)


def test_score_self_fp32_inputs_and_block_boundaries():
    """fp32 inputs are rounded to bf16 on entry; lengths at and around the 256-key / 128-query tile sizes."""
    base = synth.scaled_case(synth.CASES["llama_8k"], name="self_f32", L_s=1, H_q=2, H_kv=1, d=64, L_l=1, H_l=2, N=8, N_q=8, chunk=8,
                             n_planted=0)
    ctx = _ctx(base)
    for N in (1, 2, 127, 128, 129, 255, 256, 257, 513):
        g = torch.Generator().manual_seed(N)
        q = torch.randn(1, 2, N, 64, generator=g)
        k = torch.randn(1, 1, N, 64, generator=g)
        ref = oracle.score_self(q, k)                   # the oracle rounds to bf16 itself
        x = pk.proxykv_score_self(ctx, q.cuda(), k.cuda())
        torch.cuda.synchronize()
        assert_close(x, ref, f"score_self fp32 N={N}")


@pytest.mark.parametrize("N,N_q,chunk", [(1, 1, 1), (1, 300, 100), (129, 1, 5), (2, 130, 1000), (513, 257, 256)])
def test_score_degenerate_shapes(N, N_q, chunk):
    """One context key, one query, a chunk longer than the query axis, lengths one past the tile sizes; max and sum forms."""
    case = synth.scaled_case(synth.CASES["llama_8k"], name=f"deg_{N}_{N_q}", L_s=1, H_q=4, H_kv=2, d=64, L_l=1, H_l=2, N=N, N_q=N_q,
                             chunk=chunk, n_planted=0)
    q, kc, kr = synth.make_proxy_qk(case)
    for reduce, code in (("max", pk.PROXYKV_REDUCE_MAX), ("sum", pk.PROXYKV_REDUCE_SUM)):
        cfg = pk.config_for_case(case)
        cfg.reduce = code
        ctx = pk.proxykv_create(cfg)
        x = pk.proxykv_score(ctx, q.cuda(), kc.cuda(), kr.cuda(), chunk)
        torch.cuda.synchronize()
        assert_close(x, oracle.score(q.double(), kc.double(), kr.double(), chunk, reduce=reduce), f"score {reduce} N={N} N_q={N_q}")
        pk.proxykv_destroy(ctx)


@pytest.mark.parametrize("scale", [8.0, 30.0])
def test_score_large_logits(scale):
    """Inputs scaled up until the softmax rows are nearly one-hot (logits of several hundred): the running reference of
    pass 1 is replaced many times, probabilities are either about one or far below the absolute tolerance."""
    case = _score_case("d64_ragged")
    q, kc, kr = synth.make_proxy_qk(case)
    q, kc, kr = (q.float() * scale).to(torch.bfloat16), (kc.float() * scale).to(torch.bfloat16), (kr.float() * scale).to(torch.bfloat16)
    for reduce, code in (("max", pk.PROXYKV_REDUCE_MAX), ("sum", pk.PROXYKV_REDUCE_SUM)):
        cfg = pk.config_for_case(case)
        cfg.reduce = code
        ctx = pk.proxykv_create(cfg)
        x = pk.proxykv_score(ctx, q.cuda(), kc.cuda(), kr.cuda(), case.chunk)
        torch.cuda.synchronize()
        assert_close(x, oracle.score(q.double(), kc.double(), kr.double(), case.chunk, reduce=reduce), f"score {reduce} x{scale}")
        pk.proxykv_destroy(ctx)
    xs = pk.proxykv_score_self(_ctx(case), q.cuda(), kr.cuda())
    torch.cuda.synchronize()
    assert_close(xs, oracle.score_self(q.double(), kr.double()), f"score_self x{scale}")


def test_score_tiny_case_fp32_inputs_and_planted_keys():
    case = synth.CASES["tiny"]
    q, kc, kr = synth.make_proxy_qk(case)
    assert q.dtype == torch.float32
    ref = oracle.score(q, kc, kr, case.chunk)          # the oracle rounds the inputs to bf16 itself
    ctx = _ctx(case)
    x = pk.proxykv_score(ctx, q.cuda(), kc.cuda(), kr.cuda(), case.chunk)
    torch.cuda.synchronize()
    assert_close(x, ref, "score[tiny]")
    plan = synth.plant_plan(case)
    K = pk.proxykv_keep_count(case.N, 0.3)
    kept = pk.proxykv_topk(ctx, x, K).cpu()
    for l in range(case.L_s):
        for h in range(case.H_kv):
            assert set(plan["pos"][l, h].tolist()) <= set(kept[l, h].tolist())
            assert bool((x[l, h].cpu()[plan["pos"][l, h]] > 0.5).all())


def test_score_uniform_rows_closed_form():
    """Zero queries: every row is uniform and the score is exactly 1/(N+1)."""
    case = synth.scaled_case(_score_case("d64_ragged"), n_planted=0)
    q, kc, kr = synth.make_proxy_qk(case)
    ctx = _ctx(case)
    x = pk.proxykv_score(ctx, torch.zeros_like(q).cuda(), kc.cuda(), kr.cuda(), case.chunk)
    torch.cuda.synchronize()
    torch.testing.assert_close(x.cpu(), torch.full_like(x.cpu(), 1.0 / (case.N + 1)), rtol=1e-5, atol=0)


# ----------------------------------------------------------------------------------------------
# mapper
# ----------------------------------------------------------------------------------------------

MAP_CASES = {
    "one_window": dict(L_s=1, H_kv=2, H_q=4, L_l=1, H_l=4, N=512),
    "two_windows_ragged": dict(L_s=2, H_kv=8, H_q=8, L_l=3, H_l=8, N=2500),
    "three_windows_short_tail": dict(L_s=1, H_kv=2, H_q=2, L_l=2, H_l=4, N=3100),
}


@pytest.mark.parametrize("name", list(MAP_CASES))
def test_mapper_matches_oracle(name):
    case = synth.scaled_case(synth.CASES["llama_8k"], name=name, N_q=64, chunk=64, n_planted=0, **MAP_CASES[name])
    w = synth.make_mapper_weights(case.H_kv, case.H_l)
    g = torch.Generator().manual_seed(17)
    # score-like input: mostly small positive values with a few near one
    X = torch.rand(case.L_s, case.H_kv, case.N, generator=g) ** 8
    X = X.to(torch.float32)
    ref = oracle.mapper(X, w, case.L_l)
    ctx = _ctx(case, w)
    y = pk.proxykv_map(ctx, X.cuda())
    torch.cuda.synchronize()
    assert_close(y, ref, f"map[{name}]")
    pairing = pk.proxykv_layer_pairing(ctx.cfg)
    for a in range(case.L_l):
        for b in range(a + 1, case.L_l):
            if pairing[a] == pairing[b]:
                assert torch.equal(y[a], y[b])


@pytest.mark.parametrize("N", [1, 2, 65, 2049])
def test_mapper_degenerate_lengths(N):
    """One token, two tokens, just over one MFMA key tile, and one token past the first window (a second window of 1025)."""
    case = synth.scaled_case(synth.CASES["llama_8k"], name=f"len{N}", L_s=2, H_kv=2, H_q=2, L_l=2, H_l=4, N=N, N_q=1, chunk=1,
                             n_planted=0)
    w = synth.make_mapper_weights(case.H_kv, case.H_l)
    g = torch.Generator().manual_seed(100 + N)
    X = (torch.rand(case.L_s, case.H_kv, N, generator=g) ** 8).to(torch.float32)
    ctx = _ctx(case, w)
    y = pk.proxykv_map(ctx, X.cuda())
    torch.cuda.synchronize()
    assert_close(y, oracle.mapper(X, w, case.L_l), f"map N={N}")
    pk.proxykv_destroy(ctx)


def test_mapper_with_scores_beyond_the_half_range():
    """Sum-form scores with an attention sink (Sec. 3 prints the feature as a sum over the query axis, so one key can
    collect a share of every row): the first conv block's output reaches 1.4e5, beyond what IEEE half holds.  The
    library stores that operand as a half value times a power of two taken from the layer's largest score; the oracle
    rounds it to an 11-bit significand without a range limit.  Also the same mapper on ordinary scores right after
    (the range exponent is per call and per layer)."""
    case = synth.scaled_case(synth.CASES["llama_8k"], name="sink", L_s=2, H_kv=2, H_q=2, L_l=2, H_l=4, N=700, N_q=1, chunk=1,
                             n_planted=0)
    w = synth.make_mapper_weights(case.H_kv, case.H_l)
    g = torch.Generator().manual_seed(5)
    X = (torch.rand(case.L_s, case.H_kv, case.N, generator=g) * 8).to(torch.float32)
    X[0, :, 0] = 1.0e5                                   # layer 0: a sink at the first token and a smaller one mid-way
    X[0, :, 350] = 3.0e4
    ref = oracle.mapper(X, w, case.L_l)
    assert bool(torch.isfinite(ref).all())
    a1 = torch.nn.functional.conv1d(X[0:1].double(), w["stem.conv1.weight"].double(), w["stem.conv1.bias"].double(), padding=1)
    assert float(a1.abs().max()) > 65504.0                # the case does leave half's range
    ctx = _ctx(case, w)
    y = pk.proxykv_map(ctx, X.cuda())
    torch.cuda.synchronize()
    assert_close(y, ref, "map with a sink")
    X2 = (torch.rand(case.L_s, case.H_kv, case.N, generator=g) ** 8).to(torch.float32)
    y2 = pk.proxykv_map(ctx, X2.cuda())
    torch.cuda.synchronize()
    assert_close(y2, oracle.mapper(X2, w, case.L_l), "map after a sink")
    pk.proxykv_destroy(ctx)


def test_mapper_context_reuse_across_lengths():
    """One context called with a short, a longer and again a shorter sequence (the workspace of every lane grows in
    between; three distinct proxy layers run side by side): same bits as a fresh context each time, and the oracle's
    values on the last one."""
    case = synth.scaled_case(synth.CASES["llama_8k"], name="reuse", L_s=3, H_kv=2, H_q=2, L_l=3, H_l=4, N=700, N_q=64, chunk=64,
                             n_planted=0)
    w = synth.make_mapper_weights(case.H_kv, case.H_l)
    g = torch.Generator().manual_seed(23)
    ctx = _ctx(case, w)
    for N in (700, 2300, 300):
        X = (torch.rand(case.L_s, case.H_kv, N, generator=g) ** 8).to(torch.float32)
        y = pk.proxykv_map(ctx, X.cuda())
        fresh = _ctx(case, w)
        y_fresh = pk.proxykv_map(fresh, X.cuda())
        torch.cuda.synchronize()
        assert torch.equal(y, y_fresh), N
        pk.proxykv_destroy(fresh)
    assert_close(y, oracle.mapper(X, w, case.L_l), "map after reuse, N=300")
    pk.proxykv_destroy(ctx)


# ----------------------------------------------------------------------------------------------
# whole path
# ----------------------------------------------------------------------------------------------

def _band_check(y_ref: torch.Tensor, idx_gpu: torch.Tensor, K: int):
    """Every token whose oracle score clears the K-th score by more than the tolerance is kept, every
    token that misses it by more than the tolerance is dropped; exact equality when the K-th and
    (K+1)-th oracle scores are further apart than the tolerance."""
    rows, N = y_ref.shape
    exact = 0
    for r in range(rows):
        srt = torch.sort(y_ref[r], descending=True).values
        sK = float(srt[K - 1])
        tau = 2.0 * (ATOL + RTOL * abs(sK))
        kept = torch.zeros(N, dtype=torch.bool)
        kept[idx_gpu[r].long()] = True
        assert int(kept.sum()) == K and bool((idx_gpu[r][1:] > idx_gpu[r][:-1]).all())
        assert bool(kept[y_ref[r] > sK + tau].all()), f"row {r}: a clearly-in token was dropped"
        assert not bool(kept[y_ref[r] < sK - tau].any()), f"row {r}: a clearly-out token was kept"
        if K < N and float(srt[K - 1] - srt[K]) > tau:
            ref_idx = oracle.topk(y_ref[r:r + 1].float(), K)[0]
            assert torch.equal(idx_gpu[r].cpu(), ref_idx)
            exact += 1
    return exact


def test_prune_tiny_case_end_to_end():
    case = synth.CASES["tiny"]
    q, kc, kr = synth.make_proxy_qk(case)
    k_t, v_t = synth.make_target_kv(case)
    w = synth.make_mapper_weights(case.H_kv, case.H_l)
    X_ref, Y_ref, idx_ref, K_ref, V_ref = oracle.prune(q, kc, kr, case.chunk, 0.3, w, k_t, v_t)
    ctx = _ctx(case, w)
    x = torch.empty(case.L_s, case.H_kv, case.N, dtype=torch.float32, device="cuda")
    y = torch.empty(case.L_l, case.H_l, case.N, dtype=torch.float32, device="cuda")
    k_out, v_out, idx, K = pk.proxykv_prune(ctx, q.cuda(), kc.cuda(), kr.cuda(), case.chunk, 0.3, k_t.cuda(), v_t.cuda(),
                                            x_out=x, yhat_out=y)
    torch.cuda.synchronize()
    assert K == 153 == idx_ref.shape[-1]
    assert_close(x, X_ref, "prune.x")
    assert_close(y, Y_ref, "prune.yhat")
    _band_check(Y_ref.view(-1, case.N), idx.cpu().view(-1, K), K)
    # given the GPU's own scores, selection and compaction are exact
    idx_same = oracle.topk(y.cpu().view(-1, case.N), K).view(case.L_l, case.H_l, K)
    assert torch.equal(idx.cpu(), idx_same)
    assert torch.equal(k_out.cpu().view(torch.int16), oracle.compact(k_t, idx_same).view(torch.int16))
    assert torch.equal(v_out.cpu().view(torch.int16), oracle.compact(v_t, idx_same).view(torch.int16))
    # a second call on the same context gives the same bits
    k2, v2, idx2, _ = pk.proxykv_prune(ctx, q.cuda(), kc.cuda(), kr.cuda(), case.chunk, 0.3, k_t.cuda(), v_t.cuda())
    torch.cuda.synchronize()
    assert torch.equal(idx2, idx) and torch.equal(k2.view(torch.int16), k_out.view(torch.int16))


def test_prune_with_the_sum_form_equals_its_stages():
    """reduce = SUM through the fused call: same bits as score -> map -> top-k -> compact called one by one."""
    case = synth.scaled_case(synth.CASES["llama_8k"], name="prune_sum", L_s=2, H_q=4, H_kv=2, d=64, L_l=3, H_l=2, N=700, N_q=500,
                             chunk=200, n_planted=4)
    q, kc, kr = synth.make_proxy_qk(case, device="cuda")
    k_t, v_t = synth.make_target_kv(case, device="cuda")
    w = synth.make_mapper_weights(case.H_kv, case.H_l)
    cfg = pk.config_for_case(case)
    cfg.reduce = pk.PROXYKV_REDUCE_SUM
    ctx = pk.proxykv_create(cfg)
    pk.proxykv_set_mapper_weights(ctx, w)
    x = torch.empty(case.L_s, case.H_kv, case.N, dtype=torch.float32, device="cuda")
    y = torch.empty(case.L_l, case.H_l, case.N, dtype=torch.float32, device="cuda")
    k_out, v_out, idx, K = pk.proxykv_prune(ctx, q, kc, kr, case.chunk, 0.25, k_t, v_t, x_out=x, yhat_out=y)
    torch.cuda.synchronize()
    x2 = pk.proxykv_score(ctx, q, kc, kr, case.chunk)
    y2 = pk.proxykv_map(ctx, x2)
    idx2 = pk.proxykv_topk(ctx, y2.view(-1, case.N), K).view(case.L_l, case.H_l, K)
    k2, v2 = pk.proxykv_compact(ctx, k_t, v_t, idx2)
    torch.cuda.synchronize()
    assert K == 175
    assert torch.equal(x, x2) and torch.equal(y, y2) and torch.equal(idx, idx2)
    assert torch.equal(k_out.view(torch.int16), k2.view(torch.int16)) and torch.equal(v_out.view(torch.int16), v2.view(torch.int16))
    assert_close(x, oracle.score(q.double().cpu(), kc.double().cpu(), kr.double().cpu(), case.chunk, reduce="sum"), "prune sum x")
    pk.proxykv_destroy(ctx)
