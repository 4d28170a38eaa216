"""CPU oracle of the ProxyKV hot path (score -> map -> top-k -> compact).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
package; only the tests, the smoke check and the bench's cpu_baseline leg do.
The oracle shares no code with the HIP library.
"""
from .proxykv_oracle import (  # noqa: F401
    round_bf16,
    round_f16,
    round_sig11,
    keep_count,
    layer_pairing,
    window_spans,
    score,
    score_self,
    score_unit,
    softmax_rows_unit,
    softmax_row,
    stem,
    positional_encoding,
    encoder_layer,
    encoder_window,
    time_encoder,
    head_cross_attention,
    mapper_layer,
    mapper,
    topk,
    topk_pooled,
    mask,
    compact,
    prune,
)
