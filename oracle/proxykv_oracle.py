"""Plain CPU oracle of the ProxyKV hot path, written from the paper.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
bench's cpu_baseline leg.  It shares no code with the HIP library and the
product package never imports it.

Everything is PyTorch CPU in float64.  Each function cites the passage of the
paper ("ProxyKV: Cross-Model Proxy Pruning for Efficient Long-Context LLM
Inference") that it follows.  Where the paper is silent the reading taken is
stated in the docstring.

Pins (tests/test_oracle_*.py): brute-force masked attention and torch.softmax
for `score`; closed forms (uniform rows, single query), invariants (rows sum to
one, scores in [0, 1], key permutation equivariance) and planted heavy hitters;
torch.nn.Conv1d/BatchNorm1d/GELU, torch.nn.TransformerEncoder and per-token
brute force of the overlap average for the mapper stages; a Python sort for
`topk`; byte equality for `compact`.  The *reading* of the mapper's
unspecified hyper-parameters (stem width, encoder flavour, stage-3 sizes) has
nothing in the paper to be pinned to: parity unpinned against the authors'
mapper, pinned only to the definition written here.

Precision: the paper runs its models in 16-bit precision (App. B) and says
nothing about the mapper's own arithmetic.  The proxy's Q/K are bf16 values.
The reading taken for the mapper is that every matrix-product operand (GEMM,
second stem convolution, attention) is a 16-bit IEEE half (fp16) value while
sums, normalisation, softmax, GELU and the residual stream are kept wide.
Half rather than bf16 because activations are re-rounded some thirty times on
the way through the encoder: two correct implementations whose wide values
differ in the last bit round a few activations differently, and that
difference grows to the size of the rounding step itself; with bf16's 8-bit
significand this alone exceeds the tolerance asked of the mapped scores
(2e-3 + 1e-2 |ref|), with half's 11 bits it stays an order of magnitude below.
`round_operands=False` switches the operand rounding off, which is what the
library pins use.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import torch

F64 = torch.float64
Weights = Dict[str, torch.Tensor]


# --------------------------------------------------------------------------
# helpers
# --------------------------------------------------------------------------

def round_bf16(x: torch.Tensor) -> torch.Tensor:
    """Round to the nearest bf16 value (ties to even), returned as float64."""
    return x.to(torch.float32).to(torch.bfloat16).to(F64)


def round_f16(x: torch.Tensor) -> torch.Tensor:
    """Round to the nearest IEEE half value (ties to even), returned as float64."""
    return x.to(torch.float32).to(torch.float16).to(F64)


def round_sig11(x: torch.Tensor) -> torch.Tensor:
    """Round to the nearest value with an 11-bit significand (ties to even) and no
    limit on the exponent: IEEE half's precision without its range.  Equal to
    `round_f16` for magnitudes in half's normal range [2^-14, 65520)."""
    m, e = torch.frexp(x.to(F64))                      # x = m * 2^e with 0.5 <= |m| < 1
    return torch.ldexp(torch.round(m * 2048.0) / 2048.0, e)


def _maybe_round(x: torch.Tensor, on: bool, fmt: str = "f16") -> torch.Tensor:
    if not on:
        return x.to(F64)
    if fmt == "bf16":
        return round_bf16(x)
    return round_sig11(x) if fmt == "sig11" else round_f16(x)


def keep_count(N: int, keep_ratio: float) -> int:
    """Number of kept tokens per head for retention ratio rho (Sec. 3, problem
    formulation: Top-K thresholding at rho in (0, 1]).  The paper does not say
    how rho*N is made an integer; reading: floor, at least one token."""
    if not (0.0 < keep_ratio <= 1.0) or N <= 0:
        raise ValueError("keep_ratio must lie in (0, 1] and N must be positive")
    return max(1, min(N, int(math.floor(float(keep_ratio) * float(N)))))


def layer_pairing(L_s: int, L_l: int) -> List[int]:
    """Depth-proportional schedule (Sec. 4.1, design rationale): target layer
    l_l in [1, L_l] is paired with proxy layer ceil(l_l * L_s / L_l).
    Returned 0-based: entry l_l-1 holds l_s-1."""
    return [-((-(ll * L_s)) // L_l) - 1 for ll in range(1, L_l + 1)]


def window_spans(N: int, win: int = 2048, stride: int = 1024) -> List[Tuple[int, int]]:
    """Sliding windows of the time-axis encoder at inference (Sec. 4.1, stage 2:
    window `win`, stride `stride`).  Reading: windows start at multiples of the
    stride, the last one is cut at N (never shifted), and there are just enough
    windows to cover every token."""
    if N <= win:
        return [(0, N)]
    n_win = -((-(N - win)) // stride) + 1
    return [(k * stride, min(k * stride + win, N)) for k in range(n_win)]


# --------------------------------------------------------------------------
# O1  reconstruction-style importance score of the proxy
# --------------------------------------------------------------------------

def softmax_rows_unit(q: torch.Tensor, k_ctx: torch.Tensor, k_rec: torch.Tensor,
                      chunk: int) -> Tuple[torch.Tensor, torch.Tensor]:
    """Attention probabilities of one query head (Sec. 3, system overview:
    Softmax(Q K^T / sqrt(D)) per query row).

    q [N_q, d] are the reconstruction queries, k_ctx [N, d] the context keys,
    k_rec [N_q, d] the keys of the reconstruction tokens themselves.  Query i of
    chunk c = i // chunk sees all N context keys and the reconstruction keys j
    of its own chunk with j <= i.  Returns (P_ctx [N_q, N], P_rec [N_q, N_q]);
    every row of the two together sums to one.  Small inputs only.
    """
    q, k_ctx, k_rec = q.to(F64), k_ctx.to(F64), k_rec.to(F64)
    N_q, d = q.shape
    a = q @ k_ctx.T / math.sqrt(d)
    b = q @ k_rec.T / math.sqrt(d)
    i = torch.arange(N_q).view(-1, 1)
    j = torch.arange(N_q).view(1, -1)
    visible = (j <= i) & (torch.div(j, chunk, rounding_mode="floor") ==
                          torch.div(i, chunk, rounding_mode="floor"))
    b = torch.where(visible, b, torch.full_like(b, -math.inf))
    top = torch.maximum(a.max(dim=1).values, b.max(dim=1).values).view(-1, 1)
    ea, eb = torch.exp(a - top), torch.exp(b - top)
    Z = ea.sum(dim=1, keepdim=True) + eb.sum(dim=1, keepdim=True)
    return ea / Z, eb / Z


def softmax_row(q_i: torch.Tensor, k_ctx: torch.Tensor, k_rec_prefix: torch.Tensor) -> Tuple[torch.Tensor, torch.Tensor]:
    """The attention probabilities of ONE reconstruction query (Sec. 3, system
    overview: Softmax(q K^T / sqrt(D)) over the keys the query sees).

    q_i [d]; k_ctx [N, d] all context keys; k_rec_prefix [len, d] the
    reconstruction keys of the query's own chunk from the chunk's first token up
    to and including the query itself (len >= 1).  Returns (p_ctx [N], p_rec
    [len]); the two together sum to one.  This is one row of
    `softmax_rows_unit`, for checks at sizes where the whole matrix is too large.
    """
    q_i, k_ctx, k_rec_prefix = q_i.to(F64), k_ctx.to(F64), k_rec_prefix.to(F64)
    d = q_i.shape[0]
    a = (k_ctx @ q_i) / math.sqrt(d)
    b = (k_rec_prefix @ q_i) / math.sqrt(d)
    top = torch.maximum(a.max(), b.max())
    ea, eb = torch.exp(a - top), torch.exp(b - top)
    Z = ea.sum() + eb.sum()
    return ea / Z, eb / Z


def score_unit(q: torch.Tensor, k_ctx: torch.Tensor, k_rec: torch.Tensor, chunk: int,
               reduce: str = "max", max_block_bytes: int = 1 << 29) -> torch.Tensor:
    """Score of the N context keys of one (proxy layer, KV head).

    q [G, N_q, d] holds the G query heads of the group.  With p the row softmax
    of `softmax_rows_unit`, the score of context key n is the maximum of p[., n]
    over every reconstruction query and every head of the group (the
    KVZip-style reconstruction score that the proxy runs, Sec. 1 and Sec. 3).
    reduce="sum" gives instead the accumulation over the query axis printed in
    Sec. 3 (system overview), summed over the group.  Rows are evaluated in
    blocks only to bound memory; each row is computed exactly as defined.
    """
    q, k_ctx, k_rec = q.to(F64), k_ctx.to(F64), k_rec.to(F64)
    G, N_q, d = q.shape
    N = k_ctx.shape[0]
    scale = 1.0 / math.sqrt(d)
    X = torch.zeros(N, dtype=F64)
    rows_per_block = max(1, int(max_block_bytes // (8 * (N + chunk))))
    for g in range(G):
        for c0 in range(0, N_q, chunk):
            c1 = min(c0 + chunk, N_q)
            for r0 in range(c0, c1, rows_per_block):
                r1 = min(r0 + rows_per_block, c1)
                qi = q[g, r0:r1]
                a = (qi @ k_ctx.T) * scale                       # context logits
                b = (qi @ k_rec[c0:r1].T) * scale                # own-chunk prefix
                i = torch.arange(r0, r1).view(-1, 1)
                j = torch.arange(c0, r1).view(1, -1)
                b = torch.where(j <= i, b, torch.full_like(b, -math.inf))
                top = torch.maximum(a.max(dim=1).values, b.max(dim=1).values).view(-1, 1)
                ea = torch.exp(a - top)
                Z = ea.sum(dim=1, keepdim=True) + torch.exp(b - top).sum(dim=1, keepdim=True)
                p = ea / Z
                if reduce == "max":
                    X = torch.maximum(X, p.max(dim=0).values)
                elif reduce == "sum":
                    X = X + p.sum(dim=0)
                else:
                    raise ValueError(reduce)
    return X


def score(q_rec: torch.Tensor, k_ctx: torch.Tensor, k_rec: torch.Tensor, chunk: int,
          reduce: str = "max", round_inputs: bool = True) -> torch.Tensor:
    """Proxy feature X [L_s, H_kv, N] (Sec. 3: X in R^{B x L_s x H_s x N}, B = 1).

    q_rec [L_s, H_q, N_q, d], k_ctx [L_s, H_kv, N, d], k_rec [L_s, H_kv, N_q, d].
    Query head h reads KV head h // G (contiguous groups; the paper is silent,
    this is the Llama/Qwen convention).  Inputs are taken post-RoPE.  With
    round_inputs the inputs are first rounded to bf16, the precision the proxy
    runs in.
    """
    L_s, H_q, N_q, d = q_rec.shape
    H_kv, N = k_ctx.shape[1], k_ctx.shape[2]
    if H_q % H_kv:
        raise ValueError("H_q must be a multiple of H_kv")
    G = H_q // H_kv
    X = torch.empty(L_s, H_kv, N, dtype=F64)
    for l in range(L_s):
        for h in range(H_kv):
            X[l, h] = score_unit(_maybe_round(q_rec[l, h * G:(h + 1) * G], round_inputs, "bf16"),
                                 _maybe_round(k_ctx[l, h], round_inputs, "bf16"),
                                 _maybe_round(k_rec[l, h], round_inputs, "bf16"), chunk, reduce)
    return X


def score_self(q: torch.Tensor, k: torch.Tensor, round_inputs: bool = True, rows_per_block: int = 1024) -> torch.Tensor:
    """The proxy feature exactly as Sec. 3 (system overview) prints it: the
    post-softmax attention of the proxy's OWN prefill accumulated over the query
    axis, X[l, h, n] = sum_q Softmax(Q K^T / sqrt(d))[l, h, q, n].

    q [L_s, H_q, N, d], k [L_s, H_kv, N, d]; returns X [L_s, H_kv, N].
    Readings: the proxy is a decoder, so its prefill attention is causal (query
    q sees keys n <= q); with grouped-query attention the G query heads that
    read KV head h are summed as well, which gives the H_s = KV heads of the
    problem formulation.  Rows are evaluated in blocks only to bound memory.
    """
    L_s, H_q, N, d = q.shape
    H_kv = k.shape[1]
    if H_q % H_kv:
        raise ValueError("H_q must be a multiple of H_kv")
    G = H_q // H_kv
    scale = 1.0 / math.sqrt(d)
    X = torch.zeros(L_s, H_kv, N, dtype=F64)
    cols = torch.arange(N).view(1, -1)
    for l in range(L_s):
        for h in range(H_q):
            qh = _maybe_round(q[l, h], round_inputs, "bf16")
            kh = _maybe_round(k[l, h // G], round_inputs, "bf16")
            for r0 in range(0, N, rows_per_block):
                r1 = min(r0 + rows_per_block, N)
                logits = (qh[r0:r1] @ kh.T) * scale
                rows = torch.arange(r0, r1).view(-1, 1)
                logits = torch.where(cols <= rows, logits, torch.full_like(logits, -math.inf))
                X[l, h // G] += torch.softmax(logits, dim=1).sum(dim=0)
    return X


# --------------------------------------------------------------------------
# O2  HybridAxialMapper forward
# --------------------------------------------------------------------------

def _gelu(x: torch.Tensor) -> torch.Tensor:
    return 0.5 * x * (1.0 + torch.special.erf(x / math.sqrt(2.0)))


def _batchnorm_eval(x: torch.Tensor, w: Weights, name: str, eps: float = 1e-5) -> torch.Tensor:
    """Inference-mode batch normalisation over the channel axis of x [C, N]."""
    g, b = w[name + ".gamma"].to(F64), w[name + ".beta"].to(F64)
    mu, var = w[name + ".mean"].to(F64), w[name + ".var"].to(F64)
    return (x - mu[:, None]) / torch.sqrt(var[:, None] + eps) * g[:, None] + b[:, None]


def _conv1d_k3(u: torch.Tensor, weight: torch.Tensor, bias: torch.Tensor) -> torch.Tensor:
    """Conv1D with kernel 3, zero padding 1 along time.  u [C_in, N],
    weight [C_out, C_in, 3]: out[c, t] = bias[c] + sum_{h, tau} weight[c, h, tau] * u[h, t + tau - 1]."""
    C_in, N = u.shape
    padded = torch.zeros(C_in, N + 2, dtype=F64)
    padded[:, 1:N + 1] = u
    out = bias.to(F64)[:, None].expand(weight.shape[0], N).clone()
    for tau in range(3):
        out = out + weight[:, :, tau].to(F64) @ padded[:, tau:tau + N]
    return out


def stem(U: torch.Tensor, w: Weights, round_operands: bool = True) -> torch.Tensor:
    """Stage 1, temporal feature extraction (Sec. 4.1, Eq. 2): two stacked
    Conv1D(k=3, p=1) -> BatchNorm -> GELU blocks along time.  U [H_s, N] is one
    proxy layer's score; returns Z_local transposed to [N, D_time].

    Readings: channel widths H_s -> C_1 -> D_time with C_1 given by the weights;
    BatchNorm in inference mode with stored statistics, eps 1e-5; GELU in its
    exact erf form; the convolution runs once over the whole sequence.  The
    first convolution works on the raw fp32 scores; the second one is a matrix
    product and takes half-precision operands.  The feature of Sec. 3 in its
    sum form is not bounded by one (an attention sink collects a share of every
    query row, up to G * N_q in total), so the first block's output can leave
    half's exponent range; what the reading fixes for this operand is its
    precision (an 11-bit significand), not its range: an implementation holds it
    as a half value times a power of two of its choosing.
    """
    U = U.to(F64)
    a1 = _conv1d_k3(U, w["stem.conv1.weight"], w["stem.conv1.bias"])
    h1 = _gelu(_batchnorm_eval(a1, w, "stem.bn1"))
    h1 = _maybe_round(h1, round_operands, "sig11")
    w2 = _maybe_round(w["stem.conv2.weight"], round_operands)
    a2 = _conv1d_k3(h1, w2, w["stem.conv2.bias"])
    z = _gelu(_batchnorm_eval(a2, w, "stem.bn2"))
    return z.T.contiguous()


def positional_encoding(P: int, D: int) -> torch.Tensor:
    """Sinusoidal positional encoding (Sec. 4.1, stage 2): PE[p, 2i] =
    sin(p / 10000^(2i/D)), PE[p, 2i+1] = cos(p / 10000^(2i/D))."""
    pos = torch.arange(P, dtype=F64).view(-1, 1)
    i = torch.arange(0, D, 2, dtype=F64).view(1, -1)
    angle = pos / torch.pow(torch.tensor(10000.0, dtype=F64), i / D)
    pe = torch.zeros(P, D, dtype=F64)
    pe[:, 0::2] = torch.sin(angle)
    pe[:, 1::2] = torch.cos(angle)
    return pe


def _layernorm(x: torch.Tensor, gamma: torch.Tensor, beta: torch.Tensor, eps: float = 1e-5) -> torch.Tensor:
    mu = x.mean(dim=-1, keepdim=True)
    var = ((x - mu) ** 2).mean(dim=-1, keepdim=True)
    return (x - mu) / torch.sqrt(var + eps) * gamma.to(F64) + beta.to(F64)


def encoder_layer(x: torch.Tensor, w: Weights, i: int, n_heads: int = 8,
                  round_operands: bool = True) -> torch.Tensor:
    """One layer of the time-axis Transformer encoder (Sec. 4.1, stage 2) on a
    window x [T, D].  The paper gives depth, head count and FFN width only;
    reading: the standard post-norm encoder layer, x = LN(x + MHA(x)) then
    x = LN(x + FFN(x)), ReLU in the FFN, biases everywhere, LN eps 1e-5, full
    bidirectional attention inside the window, no dropout.

    Operand rounding: the inputs of the four linear maps, the q/k/v fed to the
    attention products and the (unnormalised, row-max-shifted) probabilities
    fed to the P V product are IEEE half values (see the module docstring);
    everything else is wide.
    """
    p = f"enc.{i}."
    T, D = x.shape
    dh = D // n_heads
    r = lambda t: _maybe_round(t, round_operands)
    qkv = r(x) @ r(w[p + "in_proj.weight"]).T + w[p + "in_proj.bias"].to(F64)
    qkv = r(qkv)
    q, k, v = qkv[:, :D], qkv[:, D:2 * D], qkv[:, 2 * D:]
    heads = []
    for h in range(n_heads):
        qh, kh, vh = (t[:, h * dh:(h + 1) * dh] for t in (q, k, v))
        s = (qh @ kh.T) / math.sqrt(dh)
        e = torch.exp(s - s.max(dim=1, keepdim=True).values)
        heads.append((r(e) @ vh) / e.sum(dim=1, keepdim=True))
    o = r(torch.cat(heads, dim=1))
    y = o @ r(w[p + "out_proj.weight"]).T + w[p + "out_proj.bias"].to(F64)
    x = _layernorm(x + y, w[p + "ln1.gamma"], w[p + "ln1.beta"])
    hdn = torch.relu(r(x) @ r(w[p + "ffn1.weight"]).T + w[p + "ffn1.bias"].to(F64))
    y2 = r(hdn) @ r(w[p + "ffn2.weight"]).T + w[p + "ffn2.bias"].to(F64)
    return _layernorm(x + y2, w[p + "ln2.gamma"], w[p + "ln2.beta"])


def _n_enc_layers(w: Weights) -> int:
    n = 0
    while f"enc.{n}.in_proj.weight" in w:
        n += 1
    return n


def encoder_window(z_win: torch.Tensor, w: Weights, n_heads: int = 8,
                   round_operands: bool = True) -> torch.Tensor:
    """The encoder on one window z_win [T, D]: add the positional encoding with
    positions restarting at 0 inside the window (this is what keeps positional
    indices in-distribution, Sec. 4.1 stage 2), then all encoder layers."""
    T, D = z_win.shape
    x = z_win.to(F64) + positional_encoding(T, D)
    for i in range(_n_enc_layers(w)):
        x = encoder_layer(x, w, i, n_heads, round_operands)
    return x


def time_encoder(z_local: torch.Tensor, w: Weights, n_heads: int = 8, win: int = 2048,
                 stride: int = 1024, round_operands: bool = True,
                 spans: Optional[Sequence[Tuple[int, int]]] = None) -> torch.Tensor:
    """Stage 2 at inference (Sec. 4.1): the encoder runs on sliding windows and
    Z_global[t] is the average of the encoder outputs of the windows that cover
    token t.  z_local [N, D] -> Z_global [N, D].  With `spans` only those
    windows are evaluated (rows that no given window covers come back as NaN;
    rows that a skipped window would also cover are not the full average)."""
    N, D = z_local.shape
    total = torch.zeros(N, D, dtype=F64)
    count = torch.zeros(N, 1, dtype=F64)
    for (s, e) in (window_spans(N, win, stride) if spans is None else spans):
        total[s:e] += encoder_window(z_local[s:e], w, n_heads, round_operands)
        count[s:e] += 1.0
    return total / count


def head_cross_attention(z_global: torch.Tensor, w: Weights, round_operands: bool = True) -> torch.Tensor:
    """Stage 3, head-axis cross-attention (Sec. 4.1, Eq. 3).  Per token t the
    latent z_t is projected to H_s key and value slots of width D_head; the
    learnable target queries Q_l [H_l, D_head] attend over the H_s slots,
    O = Softmax(Q_l K^T / sqrt(D_head)) V, and a linear map D_head -> 1 gives the
    score.  Returns the raw logit Y_hat [H_l, N] (the sigmoid of Sec. 4.2 is
    monotone, so the Top-K is the same).  Readings: D_head and H_s follow from
    the weight shapes; projections carry biases.  The two projections are matrix
    products with half-precision operands; the per-token attention is wide."""
    N, D = z_global.shape
    Ql = w["head.queries"].to(F64)
    H_l, dh = Ql.shape
    r = lambda t: _maybe_round(t, round_operands)
    K = r(z_global) @ r(w["head.k_proj.weight"]).T + w["head.k_proj.bias"].to(F64)
    V = r(z_global) @ r(w["head.v_proj.weight"]).T + w["head.v_proj.bias"].to(F64)
    H_s = K.shape[1] // dh
    K = K.view(N, H_s, dh)
    V = V.view(N, H_s, dh)
    logits = torch.einsum("he,tse->ths", Ql, K) / math.sqrt(dh)
    A = torch.softmax(logits, dim=-1)
    O = torch.einsum("ths,tse->the", A, V)
    y = torch.einsum("the,e->th", O, w["head.out.weight"].to(F64)) + w["head.out.bias"].to(F64)
    return y.T.contiguous()


def mapper_layer(U: torch.Tensor, w: Weights, n_heads: int = 8, win: int = 2048, stride: int = 1024,
                 round_operands: bool = True) -> torch.Tensor:
    """One forward of the mapper on one proxy layer's scores U [H_s, N] ->
    Y_hat [H_l, N] (Sec. 4.1: stem, windowed time-axis encoder, head-axis
    cross-attention; the raw X is fed in without any transform)."""
    z_local = stem(U, w, round_operands)
    z_global = time_encoder(z_local, w, n_heads, win, stride, round_operands)
    return head_cross_attention(z_global, w, round_operands)


def mapper(X: torch.Tensor, w: Weights, L_l: int, n_heads: int = 8, win: int = 2048, stride: int = 1024,
           round_operands: bool = True, layers: Optional[Sequence[int]] = None) -> torch.Tensor:
    """Y_hat [L_l, H_l, N] from X [L_s, H_s, N]: one mapper forward per target
    layer with shared weights, fed with the paired proxy layer, outputs stacked
    along the layer axis (Sec. 4.1, design rationale).  `layers` restricts the
    (0-based) target layers that are evaluated; the others come back as NaN."""
    L_s, H_s, N = X.shape
    H_l = w["head.queries"].shape[0]
    pairing = layer_pairing(L_s, L_l)
    Y = torch.full((L_l, H_l, N), math.nan, dtype=F64)
    for ll in (range(L_l) if layers is None else layers):
        Y[ll] = mapper_layer(X[pairing[ll]], w, n_heads, win, stride, round_operands)
    return Y


# --------------------------------------------------------------------------
# O3  per-head Top-K selection,  O4  compaction
# --------------------------------------------------------------------------

def topk(scores: torch.Tensor, K: int) -> torch.Tensor:
    """Kept-token indices [rows, K], ascending, for scores [rows, N] (Sec. 3:
    the mask M keeps the Top-K of Y_hat per layer and head).  Total order: higher
    score first, ties to the lower index; -0.0 equals +0.0; NaN ranks below
    every number.  Under a total order the kept set is unique."""
    rows, N = scores.shape
    if not (1 <= K <= N):
        raise ValueError("K must lie in [1, N]")
    s = scores.to(F64)
    isnan = torch.isnan(s)
    s = torch.where(isnan, torch.full_like(s, -math.inf), s)
    out = torch.empty(rows, K, dtype=torch.int32)
    for r in range(rows):
        # stable sorts applied from the least to the most significant key
        order = torch.arange(N)
        order = order[torch.sort(-s[r][order], stable=True).indices]
        order = order[torch.sort(isnan[r][order].to(torch.int8), stable=True).indices]
        out[r] = torch.sort(order[:K]).values.to(torch.int32)
    return out


def topk_pooled(scores: torch.Tensor, K_per_head: int) -> Tuple[torch.Tensor, torch.Tensor]:
    """Non-uniform head budgets: one selection per target layer over the pooled
    scores of all its heads (the paper thresholds Y_hat at a retention ratio,
    Sec. 3, and leaves open whether the budget is per head or shared; KVZip,
    whose score the proxy imitates, shares it across heads).  scores [L, H, N];
    the H*K_per_head best (head, token) pairs of a layer are kept under the total
    order of `topk` applied to the row of length H*N (higher score first, ties to
    the lower flat index h*N + n).  Returns (flat [L, H*K_per_head] int32, the kept
    flat indices ascending, so head h's tokens are the entries in [h*N, (h+1)*N)
    minus h*N, ascending; counts [L, H] int32, the number kept per head)."""
    L, H, N = scores.shape
    flat = topk(scores.reshape(L, H * N), H * K_per_head)
    counts = torch.zeros(L, H, dtype=torch.int32)
    for l in range(L):
        counts[l] = torch.bincount(torch.div(flat[l].to(torch.int64), N, rounding_mode="floor"), minlength=H).to(torch.int32)
    return flat, counts


def mask(idx: torch.Tensor, N: int) -> torch.Tensor:
    """The binary mask M of Sec. 3 (M in {0,1}^{B x L_l x H_l x N}) from the kept
    indices idx [..., K]: M[..., n] = 1 exactly for the kept tokens.  uint8."""
    M = torch.zeros(*idx.shape[:-1], N, dtype=torch.uint8)
    M.scatter_(-1, idx.to(torch.int64), torch.ones(idx.shape, dtype=torch.uint8))
    return M


def compact(kv: torch.Tensor, idx: torch.Tensor) -> torch.Tensor:
    """Apply the mask to a KV tensor (Sec. 3 and Sec. 4.3): kv [..., N, D] and
    idx [..., K] -> out [..., K, D] with out[..., j, :] = kv[..., idx[..., j], :].
    The kept tokens stay in their original order because idx is ascending."""
    D = kv.shape[-1]
    gather_index = idx.to(torch.int64).unsqueeze(-1).expand(*idx.shape, D)
    return torch.gather(kv, -2, gather_index)


def prune(q_rec: torch.Tensor, k_ctx: torch.Tensor, k_rec: torch.Tensor, chunk: int, keep_ratio: float,
          w: Weights, k_t: torch.Tensor, v_t: torch.Tensor, n_heads: int = 8, win: int = 2048,
          stride: int = 1024):
    """The whole path: score -> map -> Top-K -> compact.  k_t, v_t are the target
    cache [L_l, H_l, N, D].  Returns (X, Y_hat, idx, K_out, V_out)."""
    L_l, H_l, N, D = k_t.shape
    X = score(q_rec, k_ctx, k_rec, chunk)
    Y = mapper(X, w, L_l, n_heads, win, stride)
    K = keep_count(N, keep_ratio)
    idx = topk(Y.to(torch.float32).view(L_l * H_l, N), K).view(L_l, H_l, K)
    return X, Y, idx, compact(k_t, idx), compact(v_t, idx)
