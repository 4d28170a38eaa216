"""Pins of the mapper oracle (CPU only): each stage against the matching
PyTorch library module in float64 with operand rounding switched off, the
windowing against per-token brute force, stage 3 against closed forms."""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2605_16360_amd import synth

SMALL = synth.MapperDims(d_time=32, c_mid=16, n_enc_layers=2, n_enc_heads=4, d_ffn=64, d_head_x=8, win=8, stride=4)


def _w64(H_s, H_l, dims=SMALL, seed=11):
    return {k: v.to(torch.float64) for k, v in synth.make_mapper_weights(H_s, H_l, dims, seed).items()}


def test_stem_matches_conv1d_batchnorm_gelu_modules():
    H_s, N = 3, 29
    w = _w64(H_s, 5)
    U = torch.rand(H_s, N, dtype=torch.float64, generator=torch.Generator().manual_seed(1))
    layers = []
    for i, (cin, cout) in enumerate([(H_s, SMALL.c_mid), (SMALL.c_mid, SMALL.d_time)], start=1):
        conv = torch.nn.Conv1d(cin, cout, kernel_size=3, padding=1).double()
        bn = torch.nn.BatchNorm1d(cout, eps=1e-5).double()
        with torch.no_grad():
            conv.weight.copy_(w[f"stem.conv{i}.weight"]); conv.bias.copy_(w[f"stem.conv{i}.bias"])
            bn.weight.copy_(w[f"stem.bn{i}.gamma"]); bn.bias.copy_(w[f"stem.bn{i}.beta"])
            bn.running_mean.copy_(w[f"stem.bn{i}.mean"]); bn.running_var.copy_(w[f"stem.bn{i}.var"])
        layers += [conv, bn, torch.nn.GELU()]
    net = torch.nn.Sequential(*layers).eval()
    with torch.no_grad():
        ref = net(U[None])[0].T
    out = oracle.stem(U, w, round_operands=False)
    assert out.shape == (N, SMALL.d_time)
    torch.testing.assert_close(out, ref, rtol=1e-11, atol=1e-13)


def _torch_encoder(w, dims):
    layer = torch.nn.TransformerEncoderLayer(dims.d_time, dims.n_enc_heads, dims.d_ffn, dropout=0.0,
                                             activation="relu", batch_first=True, norm_first=False)
    enc = torch.nn.TransformerEncoder(layer, dims.n_enc_layers, enable_nested_tensor=False).double().eval()
    with torch.no_grad():
        for i, l in enumerate(enc.layers):
            p = f"enc.{i}."
            l.self_attn.in_proj_weight.copy_(w[p + "in_proj.weight"]); l.self_attn.in_proj_bias.copy_(w[p + "in_proj.bias"])
            l.self_attn.out_proj.weight.copy_(w[p + "out_proj.weight"]); l.self_attn.out_proj.bias.copy_(w[p + "out_proj.bias"])
            l.linear1.weight.copy_(w[p + "ffn1.weight"]); l.linear1.bias.copy_(w[p + "ffn1.bias"])
            l.linear2.weight.copy_(w[p + "ffn2.weight"]); l.linear2.bias.copy_(w[p + "ffn2.bias"])
            l.norm1.weight.copy_(w[p + "ln1.gamma"]); l.norm1.bias.copy_(w[p + "ln1.beta"])
            l.norm2.weight.copy_(w[p + "ln2.gamma"]); l.norm2.bias.copy_(w[p + "ln2.beta"])
    return enc


def test_encoder_window_matches_transformer_encoder_module():
    T = 13
    w = _w64(2, 3)
    z = torch.randn(T, SMALL.d_time, dtype=torch.float64, generator=torch.Generator().manual_seed(2))
    enc = _torch_encoder(w, SMALL)
    with torch.no_grad():
        ref = enc((z + oracle.positional_encoding(T, SMALL.d_time))[None])[0]
    out = oracle.encoder_window(z, w, SMALL.n_enc_heads, round_operands=False)
    torch.testing.assert_close(out, ref, rtol=1e-10, atol=1e-12)


def test_positional_encoding_values():
    D = 16
    pe = oracle.positional_encoding(50, D)
    assert torch.equal(pe[0], torch.tensor([0.0, 1.0] * (D // 2), dtype=torch.float64))
    for p in (1, 7, 49):
        assert abs(float(pe[p, 0]) - math.sin(p)) < 1e-15 and abs(float(pe[p, 1]) - math.cos(p)) < 1e-15
        f = 10000.0 ** (-(D - 2) / D)
        assert abs(float(pe[p, D - 2]) - math.sin(p * f)) < 1e-15 and abs(float(pe[p, D - 1]) - math.cos(p * f)) < 1e-15
        assert abs(float(pe[p, 6]) - math.sin(p / 10000.0 ** (6 / D))) < 1e-15


@pytest.mark.parametrize("N", [8, 9, 12, 21])
def test_overlap_average_against_per_token_brute_force(N):
    """Z_global[t] = mean over the windows that contain t of that window's encoder output,
    recomputed here window by window with the library encoder."""
    w = _w64(2, 3)
    z = torch.randn(N, SMALL.d_time, dtype=torch.float64, generator=torch.Generator().manual_seed(3))
    enc = _torch_encoder(w, SMALL)
    out = oracle.time_encoder(z, w, SMALL.n_enc_heads, SMALL.win, SMALL.stride, round_operands=False)
    spans = oracle.window_spans(N, SMALL.win, SMALL.stride)
    for t in range(N):
        vals = []
        for (s, e) in spans:
            if s <= t < e:
                with torch.no_grad():
                    y = enc((z[s:e] + oracle.positional_encoding(e - s, SMALL.d_time))[None])[0]
                vals.append(y[t - s])
        assert 1 <= len(vals) <= 2
        torch.testing.assert_close(out[t], torch.stack(vals).mean(0), rtol=1e-10, atol=1e-12)
    # the last window ends at N and every window starts on a stride multiple
    assert spans[-1][1] == N and all(s % SMALL.stride == 0 for s, _ in spans)


def test_head_cross_attention_against_library_and_closed_forms():
    N, H_s, H_l = 10, 3, 5
    w = _w64(H_s, H_l)
    z = torch.randn(N, SMALL.d_time, dtype=torch.float64, generator=torch.Generator().manual_seed(4))
    y = oracle.head_cross_attention(z, w, round_operands=False)
    assert y.shape == (H_l, N)
    dh = SMALL.d_head_x
    K = torch.nn.functional.linear(z, w["head.k_proj.weight"], w["head.k_proj.bias"]).view(N, H_s, dh)
    V = torch.nn.functional.linear(z, w["head.v_proj.weight"], w["head.v_proj.bias"]).view(N, H_s, dh)
    Q = w["head.queries"][None].expand(N, H_l, dh)
    O = torch.nn.functional.scaled_dot_product_attention(Q, K, V)          # scale 1/sqrt(dh), softmax over slots
    ref = (O @ w["head.out.weight"] + w["head.out.bias"]).T
    torch.testing.assert_close(y, ref, rtol=1e-11, atol=1e-13)
    # one slot: the softmax is 1, so the score is the output map of the value whatever the queries are
    w1 = _w64(1, H_l)
    y1 = oracle.head_cross_attention(z, w1, round_operands=False)
    v1 = torch.nn.functional.linear(z, w1["head.v_proj.weight"], w1["head.v_proj.bias"])
    ref1 = (v1 @ w1["head.out.weight"] + w1["head.out.bias"])[None].expand(H_l, N)
    torch.testing.assert_close(y1, ref1, rtol=1e-12, atol=1e-14)
    # identical slots: attention weights do not matter, every target head gets the common value
    w2 = dict(w)
    for nm in ("k_proj", "v_proj"):
        w2[f"head.{nm}.weight"] = w[f"head.{nm}.weight"][:dh].repeat(H_s, 1)
        w2[f"head.{nm}.bias"] = w[f"head.{nm}.bias"][:dh].repeat(H_s)
    y2 = oracle.head_cross_attention(z, w2, round_operands=False)
    v2 = torch.nn.functional.linear(z, w2["head.v_proj.weight"][:dh], w2["head.v_proj.bias"][:dh])
    torch.testing.assert_close(y2, (v2 @ w["head.out.weight"] + w["head.out.bias"])[None].expand(H_l, N), rtol=1e-12, atol=1e-14)
    # the query bank is the only H_l-dependent parameter (Sec. 4.1, stage 3)
    wa, wb = synth.make_mapper_weights(H_s, 4, SMALL, 1), synth.make_mapper_weights(H_s, 9, SMALL, 1)
    assert [k for k in wa if wa[k].shape != wb[k].shape] == ["head.queries"]


def test_mapper_stacks_layers_by_the_pairing_schedule():
    L_s, L_l, H_s, H_l, N = 2, 5, 2, 3, 11
    w = _w64(H_s, H_l)
    X = torch.rand(L_s, H_s, N, dtype=torch.float64, generator=torch.Generator().manual_seed(5))
    Y = oracle.mapper(X, w, L_l, SMALL.n_enc_heads, SMALL.win, SMALL.stride)
    assert Y.shape == (L_l, H_l, N)
    pairing = oracle.layer_pairing(L_s, L_l)
    assert pairing == [0, 0, 1, 1, 1]
    for ll in range(L_l):
        ref = oracle.mapper_layer(X[pairing[ll]], w, SMALL.n_enc_heads, SMALL.win, SMALL.stride)
        assert torch.equal(Y[ll], ref)
    assert torch.equal(Y[0], Y[1]) and not torch.equal(Y[1], Y[2])
    part = oracle.mapper(X, w, L_l, SMALL.n_enc_heads, SMALL.win, SMALL.stride, layers=[3])
    assert torch.equal(part[3], Y[3]) and bool(torch.isnan(part[0]).all())


def test_operand_rounding_is_a_small_perturbation_and_is_applied():
    H_s, H_l, N = 2, 4, 40
    w = synth.make_mapper_weights(H_s, H_l, SMALL, 3)
    U = torch.rand(H_s, N, dtype=torch.float64, generator=torch.Generator().manual_seed(6))
    a = oracle.mapper_layer(U, w, SMALL.n_enc_heads, SMALL.win, SMALL.stride, round_operands=True)
    b = oracle.mapper_layer(U, w, SMALL.n_enc_heads, SMALL.win, SMALL.stride, round_operands=False)
    diff = float((a - b).abs().max())
    assert 0.0 < diff < 0.01
    # rounding the weights beforehand changes nothing once operand rounding is on (it is idempotent)
    wr = {k: (oracle.round_f16(v) if k.endswith("proj.weight") or "ffn" in k and k.endswith("weight")
              or k == "stem.conv2.weight" else v) for k, v in w.items()}
    c = oracle.mapper_layer(U, wr, SMALL.n_enc_heads, SMALL.win, SMALL.stride, round_operands=True)
    assert torch.equal(a, c)
    # half precision keeps 11 significant bits, ties to even
    x = torch.tensor([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 65504.0, 2.0 ** -25, 3 * 2.0 ** -25], dtype=torch.float64)
    assert oracle.round_f16(x).tolist() == [1.0, 1.0 + 2.0 ** -9, 65504.0, 0.0, 2.0 ** -23]


def test_parameter_budget_order_of_magnitude():
    """Sec. 4.1 quotes ~0.5 M / ~13 M / ~1.5 M parameters; the architecture sentence (6 layers,
    FFN 4*D_time) gives 18.9 M for the encoder.  The chosen widths must land in the same decade."""
    budget = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "mapper_budget.txt")):
        if not line.startswith("#") and line.strip():
            k, v = line.split()
            budget[k] = float(v)
    w = synth.make_mapper_weights(8, 8)
    count = lambda pre: sum(v.numel() for k, v in w.items() if k.startswith(pre)) / 1e6
    stem, enc, head = count("stem."), count("enc."), count("head.")
    assert 0.5 * budget["stem"] < stem < 2 * budget["stem"]
    assert 0.5 * budget["encoder"] < enc < 2 * budget["encoder"]
    assert 0.25 * budget["head"] < head < 2 * budget["head"]
    assert abs(enc - 18.9) < 0.1          # 6 * (4*512^2 + 2*512*2048 + biases and norms)


# ----------------------------------------------------------------------------------------------
# Operand precision of the mapper (the paper does not state it): why the oracle rounds matrix-product
# operands to IEEE half and not to bf16.
# ----------------------------------------------------------------------------------------------

def _encoder_layer_rewritten(x, w, i, rt, n_heads=8, blk=64, lazy=8.0):
    """The encoder layer of Sec. 4.1 (stage 2) written a second time, as an accelerator would run it: fp32
    accumulation everywhere, the attention as an online softmax over key blocks whose reference only moves
    when a logit exceeds it by 2^lazy (probabilities rounded relative to that reference, divided by the
    unrounded sum afterwards), torch's own layer norm.  Operands of the matrix products are rounded to `rt`
    at the same places as in oracle.encoder_layer."""
    f32 = torch.float32
    r = lambda t: t.to(f32).to(rt).to(f32)
    p = f"enc.{i}."
    T, D = x.shape
    dh = D // n_heads
    x = x.to(f32)
    qkv = r(r(x) @ r(w[p + "in_proj.weight"]).T + w[p + "in_proj.bias"])
    q, k, v = qkv[:, :D], qkv[:, D:2 * D], qkv[:, 2 * D:]
    c = math.log2(math.e) / math.sqrt(dh)
    heads = []
    for h in range(n_heads):
        qh, kh, vh = (t[:, h * dh:(h + 1) * dh] for t in (q, k, v))
        m = torch.full((T, 1), -1e30, dtype=f32)
        l = torch.zeros(T, 1, dtype=f32)
        o = torch.zeros(T, dh, dtype=f32)
        for j0 in range(0, T, blk):
            s = (qh @ kh[j0:j0 + blk].T) * c
            tm = s.max(dim=1, keepdim=True).values
            nm = torch.where(tm > m + lazy, tm, m)
            alpha = torch.exp2(m - nm)
            l, o, m = l * alpha, o * alpha, nm
            pt = torch.exp2(s - m)
            l = l + pt.sum(dim=1, keepdim=True)
            o = o + r(pt) @ vh[j0:j0 + blk]
        heads.append(o / l)
    o = r(torch.cat(heads, dim=1))
    ln = lambda t, g, b: torch.nn.functional.layer_norm(t, (D,), g, b, 1e-5)
    x = ln(x + o @ r(w[p + "out_proj.weight"]).T + w[p + "out_proj.bias"], w[p + "ln1.gamma"], w[p + "ln1.beta"])
    hdn = torch.relu(r(x) @ r(w[p + "ffn1.weight"]).T + w[p + "ffn1.bias"])
    y2 = r(hdn) @ r(w[p + "ffn2.weight"]).T + w[p + "ffn2.bias"]
    return ln(x + y2, w[p + "ln2.gamma"], w[p + "ln2.beta"])


def test_two_correct_evaluations_agree_under_half_operands_but_not_under_bf16(monkeypatch):
    """Two evaluations of the same mapper that differ only in what no reading of the paper fixes (fp64 against
    fp32 accumulation, plain against online softmax) and round the matrix-product operands at the same places.
    With bf16 operands their outputs drift apart by more than the absolute tolerance asked of the mapped scores
    (2e-3): activations are re-rounded about thirty times on the way through the six layers, values that differ in
    the last bit round differently, and the difference grows to the size of bf16's rounding step.  With IEEE half
    operands (11-bit significand, same matrix-core rate) the same two evaluations stay below a quarter of it.
    This is the ground for the oracle's half-precision reading; the library follows it."""
    import oracle.proxykv_oracle as O
    H_s, H_l, N = 8, 64, 1024
    w = synth.make_mapper_weights(H_s, H_l)
    worst = {}
    for name, rt in (("bf16", torch.bfloat16), ("f16", torch.float16)):
        monkeypatch.setattr(O, "_maybe_round", lambda x, on, fmt="f16", rt=rt: x.to(torch.float32).to(rt).to(O.F64) if on else x.to(O.F64))
        worst[name] = []
        for seed in (0, 1):
            g = torch.Generator().manual_seed(7 * N + seed)
            X = (torch.rand(H_s, N, generator=g) ** 8).to(torch.float32)
            a = O.mapper_layer(X, w)
            with monkeypatch.context() as mp:
                mp.setattr(O, "encoder_layer", lambda x, w_, i, n_heads=8, round_operands=True, rt=rt:
                           _encoder_layer_rewritten(x, w_, i, rt, n_heads).double())
                b = O.mapper_layer(X, w)
            err = (a - b).abs()
            worst[name].append((float(err.max()), float((err / (2e-3 + 1e-2 * a.abs())).max())))
    assert all(e > 2e-3 for e, _ in worst["bf16"]), worst
    assert all(r > 0.5 for _, r in worst["bf16"]), worst          # most of the allclose bound is gone too
    assert all(e < 5e-4 and r < 0.25 for e, r in worst["f16"]), worst


def test_round_sig11_is_half_precision_without_the_range():
    """The rounding of the second convolution's operand: IEEE half's values where half has them, the same
    relative spacing beyond its range (every power-of-two multiple of a representable value is representable)."""
    g = torch.Generator().manual_seed(3)
    x = torch.randn(20000, dtype=torch.float64, generator=g) * torch.pow(2.0, torch.randint(-13, 15, (20000,), generator=g).double())
    x = x[(x.abs() >= 2.0 ** -14) & (x.abs() < 65504.0)]
    assert torch.equal(oracle.round_sig11(x), oracle.round_f16(x))
    for k in (-40, -17, 5, 30):
        assert torch.equal(oracle.round_sig11(x * 2.0 ** k), oracle.round_sig11(x) * 2.0 ** k)
    big = torch.tensor([65504.0, 65519.9, 65520.0, 1.0e5, 3.0e5 + 7.0, 1.2e6, -2.5e9], dtype=torch.float64)
    r = oracle.round_sig11(big)
    assert bool(torch.isfinite(r).all()) and bool(((r - big).abs() <= big.abs() * 2.0 ** -11).all())
    assert float(r[0]) == 65504.0 and float(r[2]) == 65536.0            # ties to even: 65520 lies halfway between 65504 and 65536
    # hand values: 11 significant bits around 1 are multiples of 2^-10, ties go to the even neighbour
    hand = torch.tensor([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -10 + 2.0 ** -12, 0.0, -3.0], dtype=torch.float64)
    assert oracle.round_sig11(hand).tolist() == [1.0, 1.0 + 2.0 ** -9, 1.0 + 2.0 ** -10, 0.0, -3.0]
