"""GPU parity at the workloads' full sizes, in the launch configuration bench.py times (one
proxykv_prune over all layers), on outputs the CPU oracle can compute one by one.

Every oracle input comes from the seeded generator (synth), never from the HIP path:
  * scoring  - one whole (proxy layer, KV head) unit key by key (llama_8k, llama_32k, qwen32b_32k; at qwen_170k,
               where one unit is 2.6e13 oracle flop, all 170 000 context keys of a unit against the first 4112
               queries of its seven heads: two whole chunks and a ragged one of 16); on every
               workload the planted heavy hitters (their source query's softmax row is one matrix-vector
               product; the score lies between that probability and 1) and, for sampled queries at chunk
               starts, chunk ends and the ragged tail, the bound X[n] >= p_i(n) on all N keys at once;
  * mapper   - proxykv_map on a seeded score-like X of the full shape, against the oracle on sampled spans
               (two adjacent windows pin a fully averaged 1024-token span; the first and last windows pin
               the singly covered ends and the ragged tail) for every target layer paired with the sampled
               proxy layer;
  * top-k    - proxykv_topk on a seeded array of the full shape, every row, bit-exact;
  * compact  - proxykv_compact and proxykv_compact_inplace on the full target cache, sampled (layer, head)
               rows, bit-exact; proxykv_mask, every row.
The fused call is then tied to the stage calls: on the same inputs it returns the same bits as
score -> map -> top-k -> compact called one by one.
Floating point: |gpu - ref| <= 2e-3 + 1e-2 |ref|.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2605_16360_amd import binding as pk
from paper_2605_16360_amd import synth

pytestmark = pytest.mark.gpu
ATOL, RTOL = 2e-3, 1e-2


def _close(g: torch.Tensor, r: torch.Tensor, what: str):
    g, r = g.detach().double().cpu(), r.double()
    assert g.shape == r.shape, (what, g.shape, r.shape)
    assert bool(torch.isfinite(g).all()), f"{what}: non-finite values"
    err = (g - r).abs()
    bound = ATOL + RTOL * r.abs()
    worst = int(torch.argmax(err - bound))
    assert bool((err <= bound).all()), (f"{what}: max abs err {float(err.max()):.3e}, worst at flat {worst}: "
                                        f"gpu {float(g.flatten()[worst])} ref {float(r.flatten()[worst])}")


def _sample_queries(case, rng, n_extra=2):
    """Query indices at chunk starts, chunk ends, the ragged tail and a few random places."""
    qs = {0, min(case.chunk, case.N_q) - 1, case.N_q - 1, ((case.N_q - 1) // case.chunk) * case.chunk}
    if case.N_q > case.chunk:
        qs |= {case.chunk, 2 * case.chunk - 1 if case.N_q >= 2 * case.chunk else case.N_q - 1}
    qs |= {int(v) for v in rng.integers(0, case.N_q, size=n_extra)}
    return sorted(qs)


def _check_scores(case, x_gpu, q, kc, kr, units, full_unit=None):
    """x_gpu [L_s, H_kv, N] on the GPU; q, kc, kr the (GPU) bf16 inputs.  `units` = (layer, KV head) pairs
    checked through planted keys and row bounds; `full_unit` one pair compared key by key."""
    G, N = case.G, case.N
    plan = synth.plant_plan(case)
    rng = np.random.default_rng(5)
    x_min, x_max = float(x_gpu.min()), float(x_gpu.max())
    assert x_min >= 0.0 and x_max <= 1.0, (x_min, x_max)
    for (l, h) in units:
        kc_u, kr_u = kc[l, h].double().cpu(), kr[l, h].double().cpu()
        xg = x_gpu[l, h].double().cpu()
        # planted heavy hitters: p of the source query's row <= X <= 1
        n_pl = min(case.n_planted, 24)
        for j in range(n_pl):
            pos, g, i = int(plan["pos"][l, h, j]), int(plan["g"][l, h, j]), int(plan["i"][l, h, j])
            lo = (i // case.chunk) * case.chunk
            p_ctx, _ = oracle.softmax_row(q[l, h * G + g, i].double().cpu(), kc_u, kr_u[lo:i + 1])
            p = float(p_ctx[pos])
            assert p > 0.5, "the planted key does not dominate its source row"
            assert float(xg[pos]) >= p - (ATOL + RTOL * p), (l, h, pos, float(xg[pos]), p)
            if p > 1.0 - 1e-3:  # then [p, 1] pins the score itself
                assert abs(float(xg[pos]) - p) <= ATOL + RTOL * p
        # sampled rows: the score of every key is at least that row's probability
        for g in sorted({0, G - 1}):
            for i in _sample_queries(case, rng):
                lo = (i // case.chunk) * case.chunk
                p_ctx, _ = oracle.softmax_row(q[l, h * G + g, i].double().cpu(), kc_u, kr_u[lo:i + 1])
                slack = ATOL + RTOL * p_ctx
                bad = xg < p_ctx - slack
                assert not bool(bad.any()), (l, h, g, i, int(bad.nonzero()[0]))
    if full_unit is not None:
        l, h = full_unit
        ref = oracle.score_unit(q[l, h * G:(h + 1) * G].double().cpu(), kc[l, h].double().cpu(), kr[l, h].double().cpu(),
                                case.chunk)
        _close(x_gpu[l, h], ref, f"score[{case.name}] unit ({l}, {h})")


def _score_like(shape, seed):
    """Seeded stand-in for a score tensor: mostly small positive values, a few near one."""
    u = synth.normal_tensor(shape, seed, 31, device="cuda")
    return (torch.sigmoid(1.5 * u) ** 8).contiguous()


def _oracle_span(X_l, w, a, b, win=2048, stride=1024):
    """Oracle Y_hat[:, a:b] of one proxy layer's scores X_l [H_s, N] (CPU fp64): the stem on the span
    plus the reach of the windows that cover it, those windows' encoder passes, their average, stage 3."""
    N = X_l.shape[1]
    spans = [(s, e) for (s, e) in oracle.window_spans(N, win, stride) if s < b and e > a]
    lo, hi = min(s for s, _ in spans), max(e for _, e in spans)
    s0, s1 = max(0, lo - 2), min(N, hi + 2)          # two k = 3 convolutions reach two tokens each way
    z = oracle.stem(X_l[:, s0:s1], w)                 # [s1 - s0, D]
    # rows near a cut that is not the sequence's end are wrong within two tokens of it; they lie outside [lo, hi)
    z_local = torch.full((N, z.shape[1]), math.nan, dtype=torch.float64)
    z_local[lo:hi] = z[lo - s0:hi - s0]
    zg = torch.zeros(b - a, z.shape[1], dtype=torch.float64)
    cnt = torch.zeros(b - a, 1, dtype=torch.float64)
    for (s, e) in spans:
        out = oracle.encoder_window(z_local[s:e], w)
        u0, u1 = max(a, s), min(b, e)
        zg[u0 - a:u1 - a] += out[u0 - s:u1 - s]
        cnt[u0 - a:u1 - a] += 1.0
    return oracle.head_cross_attention(zg / cnt, w)   # [H_l, b - a]


def _check_mapper(case, ctx, w, samples):
    """samples: (proxy layer, a, b) spans."""
    X = _score_like((case.L_s, case.H_kv, case.N), 41)
    y = pk.proxykv_map(ctx, X)
    torch.cuda.synchronize()
    pairing = pk.proxykv_layer_pairing(ctx.cfg)
    for (ls, a, b) in samples:
        ref = _oracle_span(X[ls].double().cpu(), w, a, b)
        targets = [ll for ll in range(case.L_l) if pairing[ll] == ls]
        assert targets
        for ll in targets:
            _close(y[ll, :, a:b], ref, f"map[{case.name}] proxy layer {ls} -> target layer {ll}, tokens [{a}, {b})")
    return X, y


def _check_topk_compact(case, ctx, keep_ratio, rows_sampled=6):
    N, rows = case.N, case.L_l * case.H_l
    K = pk.proxykv_keep_count(N, keep_ratio)
    assert K == oracle.keep_count(N, keep_ratio)
    s = synth.normal_tensor((rows, N), 9, 51, device="cuda")
    s[1] = torch.round(s[1] * 8) / 8                   # heavy ties
    s[2] = 0.25                                        # all equal
    idx = pk.proxykv_topk(ctx, s, K)
    torch.cuda.synchronize()
    ref = oracle.topk(s.cpu(), K)
    assert torch.equal(idx.cpu(), ref), f"top-k[{case.name}] differs"
    k_t, v_t = synth.make_target_kv(case, device="cuda")
    idx_l = ref.view(case.L_l, case.H_l, K).cuda()
    k_out, v_out = pk.proxykv_compact(ctx, k_t, v_t, idx_l)
    torch.cuda.synchronize()
    rng = np.random.default_rng(11)
    picks = {(0, 0), (case.L_l - 1, case.H_l - 1)} | {(int(rng.integers(case.L_l)), int(rng.integers(case.H_l)))
                                                       for _ in range(rows_sampled - 2)}
    # the same gather with the cache as its own destination, and the byte mask
    k_ip, v_ip = k_t.clone(), v_t.clone()
    pk.proxykv_compact_inplace(ctx, k_ip, v_ip, idx_l)
    m = pk.proxykv_mask(ctx, idx_l, N)
    torch.cuda.synchronize()
    assert torch.equal(m.cpu(), oracle.mask(ref.view(case.L_l, case.H_l, K), N)), f"mask[{case.name}] differs"
    for (l, h) in sorted(picks):
        for src, out, inplace in ((k_t, k_out, k_ip), (v_t, v_out, v_ip)):
            exp = oracle.compact(src[l:l + 1, h:h + 1].cpu(), idx_l[l:l + 1, h:h + 1].cpu())
            assert torch.equal(out[l:l + 1, h:h + 1].cpu().view(torch.int16), exp.view(torch.int16)), (case.name, l, h)
            assert torch.equal(inplace[l:l + 1, h:h + 1, :K].cpu().view(torch.int16), exp.view(torch.int16)), (case.name, l, h)
            assert torch.equal(inplace[l, h, K:].view(torch.int16), src[l, h, K:].view(torch.int16)), (case.name, l, h)
    del k_ip, v_ip
    # one budget per layer shared by its heads: selection against the oracle on every layer, the ragged
    # compaction on the sampled rows
    s3 = s.view(case.L_l, case.H_l, N)
    s3[0, 0] += 1.0                                    # moves budget between the heads of layer 0
    flat, counts = pk.proxykv_topk_pooled(ctx, s3, K)
    torch.cuda.synchronize()
    flat_ref, counts_ref = oracle.topk_pooled(s3.cpu(), K)
    assert torch.equal(flat.cpu(), flat_ref) and torch.equal(counts.cpu(), counts_ref), f"pooled top-k[{case.name}] differs"
    assert int(counts_ref[0, 0]) > K
    k_pl, v_pl = k_t.clone(), v_t.clone()
    pk.proxykv_compact_pooled(ctx, k_pl, v_pl, flat, counts)
    torch.cuda.synchronize()
    starts = torch.cumsum(counts_ref, 1) - counts_ref
    for (l, h) in sorted(picks):
        c, st = int(counts_ref[l, h]), int(starts[l, h])
        tok = (flat_ref[l, st:st + c].to(torch.int64) - h * N).cuda()
        for src, got in ((k_t, k_pl), (v_t, v_pl)):
            assert torch.equal(got[l, h, :c].view(torch.int16), src[l, h][tok].view(torch.int16)), (case.name, l, h)
            assert torch.equal(got[l, h, c:].view(torch.int16), src[l, h, c:].view(torch.int16)), (case.name, l, h)
    del k_pl, v_pl
    return k_t, v_t


def _check_fused_equals_stages(case, ctx, q, kc, kr, k_t, v_t, keep_ratio):
    """proxykv_prune against the stage entry points called one by one on the same inputs: same bits."""
    dev = "cuda"
    x = torch.empty(case.L_s, case.H_kv, case.N, dtype=torch.float32, device=dev)
    y = torch.empty(case.L_l, case.H_l, case.N, dtype=torch.float32, device=dev)
    k_out, v_out, idx, K = pk.proxykv_prune(ctx, q, kc, kr, case.chunk, keep_ratio, k_t, v_t, x_out=x, yhat_out=y)
    torch.cuda.synchronize()
    # and with the Top-K kernel gathering the kept tokens itself
    pk.proxykv_set_fused_select(ctx, True)
    k_f, v_f, idx_f, _ = pk.proxykv_prune(ctx, q, kc, kr, case.chunk, keep_ratio, k_t, v_t)
    pk.proxykv_set_fused_select(ctx, False)
    torch.cuda.synchronize()
    assert torch.equal(idx_f, idx) and torch.equal(k_f.view(torch.int16), k_out.view(torch.int16))
    assert torch.equal(v_f.view(torch.int16), v_out.view(torch.int16))
    del k_f, v_f, idx_f
    x2 = pk.proxykv_score(ctx, q, kc, kr, case.chunk)
    y2 = pk.proxykv_map(ctx, x2)
    idx2 = pk.proxykv_topk(ctx, y2.view(-1, case.N), K).view(case.L_l, case.H_l, K)
    k2, v2 = pk.proxykv_compact(ctx, k_t, v_t, idx2)
    torch.cuda.synchronize()
    assert torch.equal(x, x2) and torch.equal(y, y2) and torch.equal(idx, idx2)
    assert torch.equal(k_out.view(torch.int16), k2.view(torch.int16)) and torch.equal(v_out.view(torch.int16), v2.view(torch.int16))
    assert bool((idx[..., 1:] > idx[..., :-1]).all()) and int(idx.min()) >= 0 and int(idx.max()) < case.N
    return x


def _run_case(name, units, full_unit, map_samples, keep_ratio=0.3):
    case = synth.CASES[name]
    w = synth.make_mapper_weights(case.H_kv, case.H_l)
    ctx = pk.proxykv_create(pk.config_for_case(case))
    pk.proxykv_set_mapper_weights(ctx, w)
    pk.proxykv_reserve(ctx, case.N, case.N_q)
    _check_mapper(case, ctx, w, map_samples)
    k_t, v_t = _check_topk_compact(case, ctx, keep_ratio)
    q, kc, kr = synth.make_proxy_qk(case, device="cuda")
    x = _check_fused_equals_stages(case, ctx, q, kc, kr, k_t, v_t, keep_ratio)
    _check_scores(case, x, q, kc, kr, units, full_unit)
    pk.proxykv_destroy(ctx)


def test_llama_8k_full_size():
    N = synth.CASES["llama_8k"].N
    _run_case("llama_8k", units=[(0, 0), (7, 3), (15, 7)], full_unit=(9, 5),
              map_samples=[(0, 0, 2048), (8, 3072, 4096), (15, N - 2048, N)])


def test_llama_8k_sum_form_full_size():
    """reduce = SUM at full size: one whole (layer, KV head) unit key by key; on other units the total over the
    keys against the number of query rows (a row gives the context at most all of its probability, and at least
    all but what its own chunk's prefix takes: bounded below through the first query of every chunk)."""
    case = synth.CASES["llama_8k"]
    cfg = pk.config_for_case(case)
    cfg.reduce = pk.PROXYKV_REDUCE_SUM
    ctx = pk.proxykv_create(cfg)
    q, kc, kr = synth.make_proxy_qk(case, device="cuda")
    x = pk.proxykv_score(ctx, q, kc, kr, case.chunk)
    torch.cuda.synchronize()
    G, (l, h) = case.G, (11, 6)
    ref = oracle.score_unit(q[l, h * G:(h + 1) * G].double().cpu(), kc[l, h].double().cpu(), kr[l, h].double().cpu(),
                            case.chunk, reduce="sum")
    _close(x[l, h], ref, "score sum[llama_8k] unit (11, 6)")
    tot = x.double().sum(dim=-1)
    assert float(tot.max()) <= G * case.N_q * (1 + 1e-5) and float(tot.min()) > 0.5 * G * case.N_q
    assert float(x.min()) >= 0.0
    pk.proxykv_destroy(ctx)


def test_llama_8k_sum_form_score_then_map_against_the_oracle():
    """The feature in the form Sec. 3 prints (sum over the query axis) feeding the mapper of Sec. 4.1 at full size:
    proxykv_score (reduce = SUM) then proxykv_map on the GPU, against the oracle's own scores of the sampled proxy
    layers' eight KV heads pushed through the oracle's mapper on sampled spans.  No oracle input comes from the GPU."""
    case = synth.CASES["llama_8k"]
    w = synth.make_mapper_weights(case.H_kv, case.H_l)
    cfg = pk.config_for_case(case)
    cfg.reduce = pk.PROXYKV_REDUCE_SUM
    ctx = pk.proxykv_create(cfg)
    pk.proxykv_set_mapper_weights(ctx, w)
    q, kc, kr = synth.make_proxy_qk(case, device="cuda")
    x = pk.proxykv_score(ctx, q, kc, kr, case.chunk)
    y = pk.proxykv_map(ctx, x)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(y).all())
    pairing = pk.proxykv_layer_pairing(ctx.cfg)
    G = case.G
    for (ls, a, b) in ((3, 0, 1024), (12, case.N - 1024, case.N)):
        X_l = torch.stack([oracle.score_unit(q[ls, h * G:(h + 1) * G].double().cpu(), kc[ls, h].double().cpu(),
                                             kr[ls, h].double().cpu(), case.chunk, reduce="sum") for h in range(case.H_kv)])
        _close(x[ls], X_l, f"score sum[llama_8k] proxy layer {ls}")
        ref = _oracle_span(X_l, w, a, b)
        for ll in [t for t in range(case.L_l) if pairing[t] == ls]:
            _close(y[ll, :, a:b], ref, f"sum-form score -> map[llama_8k] proxy layer {ls} -> target layer {ll}, tokens [{a}, {b})")
    pk.proxykv_destroy(ctx)


def test_llama_8k_score_self_full_size():
    """The causal self-attention feature at full size: one whole (layer, KV head) unit key by key against the oracle;
    on every unit the total over the keys equals the number of query rows (every row is a probability vector), the
    last key holds what the last query gives itself (at most one per head), and nothing is negative."""
    case = synth.CASES["llama_8k"]
    ctx = pk.proxykv_create(pk.config_for_case(case))
    q, _, k = synth.make_proxy_qk(case, device="cuda")
    x = pk.proxykv_score_self(ctx, q, k)
    torch.cuda.synchronize()
    G, (l, h) = case.G, (9, 2)
    ref = oracle.score_self(q[l:l + 1, h * G:(h + 1) * G].double().cpu(), k[l:l + 1, h:h + 1].double().cpu())[0, 0]
    _close(x[l, h], ref, "score_self[llama_8k] unit (9, 2)")
    tot = x.double().sum(dim=-1)
    assert torch.allclose(tot, torch.full_like(tot, float(G * case.N_q)), rtol=1e-4)
    assert float(x.min()) >= 0.0 and float(x[..., -1].max()) <= G * (1 + 1e-5)
    pk.proxykv_destroy(ctx)


@pytest.mark.parametrize("name,keep_ratio", [("llama_32k", 0.1), ("llama_32k", 0.5), ("qwen32b_32k", 0.9)])
def test_selection_and_compaction_at_the_other_keep_ratios(name, keep_ratio):
    """Top-K on every row, both compactions, the mask and the pooled budget at the workloads' other retention ratios."""
    case = synth.CASES[name]
    ctx = pk.proxykv_create(pk.config_for_case(case))
    k_t, v_t = _check_topk_compact(case, ctx, keep_ratio)
    del k_t, v_t
    pk.proxykv_destroy(ctx)


def test_llama_32k_full_size():
    """The workload bench.py times."""
    N = synth.CASES["llama_32k"].N
    _run_case("llama_32k", units=[(0, 0), (15, 7)], full_unit=(6, 2),
              map_samples=[(0, 0, 2048), (7, 16384, 17408), (15, N - 2048, N)])


def test_qwen32b_32k_full_size():
    """Head dimension 128, groups of 6, chunks of 4096, 64 target layers paired with 28 proxy layers."""
    N = synth.CASES["qwen32b_32k"].N
    _run_case("qwen32b_32k", units=[(0, 0), (27, 1)], full_unit=(13, 1),
              map_samples=[(0, 0, 1024), (27, N - 1024, N)], keep_ratio=0.5)


def test_qwen_170k_full_size():
    """N = 170000: ragged key tiles, a last chunk of 16 queries, 166 windows with a short tail, rows longer
    than the top-k kernel can hold in LDS."""
    N = synth.CASES["qwen_170k"].N
    _run_case("qwen_170k", units=[(0, 0), (23, 1)], full_unit=None,
              map_samples=[(0, 0, 1024), (11, 84992, 86016), (23, N - 1024, N)])


def test_qwen_170k_score_two_sided_on_all_context_keys():
    """All 170 000 context keys of one (layer, KV head) of the qwen_170k workload, groups of seven heads, against the
    oracle key by key, with the first 4112 reconstruction queries of every head (two whole chunks of 2048 and a ragged
    chunk of 16): ragged key tiles, the ragged last chunk and the group reduction at the workload's own key count.
    The whole unit (170 000 queries per head) is 2.6e13 oracle flop and is covered by bounds in the test above."""
    case = synth.CASES["qwen_170k"]
    l, h, nq = 17, 1, 2 * case.chunk + 16
    sub = synth.scaled_case(case, name="qwen_170k_unit", L_s=1, H_q=case.G, H_kv=1, L_l=1, H_l=1, N_q=nq)
    # the unit's own tensors: rows of the full workload's streams, generated unit by unit
    G, N, d = case.G, case.N, case.d
    q = torch.empty(1, G, nq, d, dtype=torch.bfloat16, device="cuda")
    for g in range(G):
        start = ((l * case.H_q + h * G + g) * case.N_q) * d
        q[0, g] = synth.irwin_hall(synth.MASTER_SEED, synth.TID_Q_REC, start, nq * d, "cuda").view(nq, d).to(torch.bfloat16)
    kc = synth.irwin_hall(synth.MASTER_SEED, synth.TID_K_CTX, ((l * case.H_kv + h) * N) * d, N * d, "cuda").view(1, 1, N, d)
    kr = synth.irwin_hall(synth.MASTER_SEED, synth.TID_K_REC, ((l * case.H_kv + h) * case.N_q) * d, nq * d, "cuda").view(1, 1, nq, d)
    # heavy hitters as in the workload: 340 context keys are three times a query of the group
    rng = np.random.default_rng(170)
    pos = rng.choice(N, size=case.n_planted, replace=False)
    src = rng.choice(G * nq, size=case.n_planted, replace=False)
    kc[0, 0, torch.from_numpy(pos).cuda()] = case.plant_scale * q[0].float().view(G * nq, d)[torch.from_numpy(src).cuda()]
    kc, kr = kc.to(torch.bfloat16).contiguous(), kr.to(torch.bfloat16).contiguous()
    for reduce, code in (("max", pk.PROXYKV_REDUCE_MAX), ("sum", pk.PROXYKV_REDUCE_SUM)):
        cfg = pk.config_for_case(sub)
        cfg.reduce = code
        ctx = pk.proxykv_create(cfg)
        x = pk.proxykv_score(ctx, q, kc, kr, case.chunk)
        torch.cuda.synchronize()
        ref = oracle.score_unit(q[0].double().cpu(), kc[0, 0].double().cpu(), kr[0, 0].double().cpu(), case.chunk, reduce=reduce)
        _close(x[0, 0], ref, f"score {reduce}[qwen_170k] unit ({l}, {h}), {nq} queries")
        if reduce == "max":
            assert float(x[0, 0, torch.from_numpy(pos).cuda()].min()) > 0.5
        pk.proxykv_destroy(ctx)


def test_qwen32b_shape_score_two_sided_mid_size():
    """Head width 128, groups of six, chunks of 4096 at N = N_q = 8192 (two chunks): every (layer, KV head) key by key,
    max and sum forms, through the same kernels and column tiling as the qwen32b_32k workload."""
    case = synth.scaled_case(synth.CASES["qwen32b_32k"], name="qwen32b_8k", L_s=2, L_l=2, N=8192, N_q=8192, n_planted=82)
    q, kc, kr = synth.make_proxy_qk(case, device="cuda")
    for reduce, code in (("max", pk.PROXYKV_REDUCE_MAX), ("sum", pk.PROXYKV_REDUCE_SUM)):
        cfg = pk.config_for_case(case)
        cfg.reduce = code
        ctx = pk.proxykv_create(cfg)
        x = pk.proxykv_score(ctx, q, kc, kr, case.chunk)
        torch.cuda.synchronize()
        ref = oracle.score(q.double().cpu(), kc.double().cpu(), kr.double().cpu(), case.chunk, reduce=reduce)
        _close(x, ref, f"score {reduce}[qwen32b shapes, 8k]")
        pk.proxykv_destroy(ctx)


def test_prune_is_bit_identical_next_to_a_busy_second_stream():
    """The paper's single-GPU regime (Sec. 4.3, App. A): the proxy side shares the device with the target's prefill
    through streams.  One proxykv_prune (which itself spreads the mapper over up to four streams the context owns) runs
    while a second stream loops large bf16 matrix products; scores, mapped scores, kept indices and the compacted
    cache must equal those of a run on a quiet device bit for bit."""
    case = synth.CASES["llama_8k"]
    w = synth.make_mapper_weights(case.H_kv, case.H_l)
    ctx = pk.proxykv_create(pk.config_for_case(case))
    pk.proxykv_set_mapper_weights(ctx, w)
    pk.proxykv_reserve(ctx, case.N, case.N_q)
    q, kc, kr = synth.make_proxy_qk(case, device="cuda")
    k_t, v_t = synth.make_target_kv(case, device="cuda")

    def run(stream):
        x = torch.empty(case.L_s, case.H_kv, case.N, dtype=torch.float32, device="cuda")
        y = torch.empty(case.L_l, case.H_l, case.N, dtype=torch.float32, device="cuda")
        k_out, v_out, idx, K = pk.proxykv_prune(ctx, q, kc, kr, case.chunk, 0.3, k_t, v_t, x_out=x, yhat_out=y, stream=stream)
        return x, y, idx, k_out, v_out

    main = torch.cuda.Stream()
    torch.cuda.synchronize()
    quiet = run(main)
    torch.cuda.synchronize()
    a = torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16)
    b = torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16)
    c = torch.empty(8192, 8192, device="cuda", dtype=torch.bfloat16)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(side):
        ev0.record(side)
        for _ in range(60):                       # about 50 ms of stand-in prefill when alone
            torch.matmul(a, b, out=c)
        ev1.record(side)
    pm0, pm1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    pm0.record(main)
    busy = run(main)
    pm1.record(main)
    torch.cuda.synchronize()
    # the two really ran at the same time: each started before the other ended (device time stamps)
    assert pm0.elapsed_time(ev1) > 0.0 and ev0.elapsed_time(pm1) > 0.0, "the two streams did not overlap in time"
    assert pm0.elapsed_time(ev1) > 5.0, "the second stream's load ended right after the prune began"
    for name, g, r in zip(("x", "yhat", "idx", "k_out", "v_out"), busy, quiet):
        same = torch.equal(g.view(torch.int16), r.view(torch.int16)) if g.dtype == torch.bfloat16 else torch.equal(g, r)
        assert same, f"{name} differs when a second stream is busy"
    pk.proxykv_destroy(ctx)
