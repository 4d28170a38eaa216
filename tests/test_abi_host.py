"""Host-side checks of the C ABI that need no GPU: the library loads and exports every symbol the
header declares, host helpers agree with the oracle, and argument validation (which runs before
any HIP call) returns the documented status codes."""
import ctypes
import os
import re

import pytest
import torch

import oracle
from paper_2605_16360_amd import binding as pk
from paper_2605_16360_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "proxykv.h")).read()
    declared = sorted(set(re.findall(r"\b(proxykv_[a-z_]+)\s*\(", header)))
    assert set(declared) == set(pk.EXPORTS)
    lib = pk.load()
    for name in declared:
        assert hasattr(lib, name), name


def test_keep_count_and_pairing_match_the_oracle():
    for N, r in [(512, 0.3), (8192, 0.3), (32768, 0.1), (32768, 0.5), (32768, 0.9), (170000, 0.3), (3, 0.1), (7, 1.0)]:
        assert pk.proxykv_keep_count(N, r) == oracle.keep_count(N, r)
    for (L_s, L_l) in [(16, 32), (24, 28), (28, 64), (1, 1), (5, 3)]:
        cfg = pk.make_config(L_s, 4, 2, 64, L_l, 4, 128)
        assert pk.proxykv_layer_pairing(cfg) == oracle.layer_pairing(L_s, L_l)
    with pytest.raises(pk.ProxyKVError) as e:
        pk.proxykv_keep_count(10, 0.0)
    assert e.value.status == pk.PROXYKV_EINVAL
    with pytest.raises(pk.ProxyKVError):
        pk.proxykv_keep_count(10, 1.5)
    with pytest.raises(pk.ProxyKVError):
        pk.proxykv_keep_count(0, 0.5)


def test_weight_blob_layout_matches_the_generator():
    for H_s, H_l in [(2, 4), (8, 8)]:
        cfg = pk.make_config(1, 2 * H_s, H_s, 64, 1, H_l, 128)
        w = synth.make_mapper_weights(H_s, H_l)
        assert set(pk.weight_names(cfg)) == set(w)
        assert pk.pack_mapper_weights(cfg, w).size == pk.proxykv_mapper_weight_count(cfg) == sum(v.numel() for v in w.values())


def test_config_validation():
    good = pk.make_config(16, 32, 8, 64, 32, 8, 128)
    ctx = pk.proxykv_create(good)
    pk.proxykv_destroy(ctx)
    for field, value, status in [("H_q", 30, pk.PROXYKV_EINVAL), ("L_s", 0, pk.PROXYKV_EINVAL),
                                 ("d", 96, pk.PROXYKV_EUNSUPPORTED), ("D", 100, pk.PROXYKV_EUNSUPPORTED),
                                 ("reduce", 7, pk.PROXYKV_EINVAL),
                                 ("d_time", 256, pk.PROXYKV_EUNSUPPORTED), ("stride", 4096, pk.PROXYKV_EINVAL)]:
        cfg = pk.make_config(16, 32, 8, 64, 32, 8, 128)
        setattr(cfg, field, value)
        with pytest.raises(pk.ProxyKVError) as e:
            pk.proxykv_create(cfg)
        assert e.value.status == status, field
        assert pk.proxykv_mapper_weight_count(cfg) == 0
    assert pk.strerror(pk.PROXYKV_EINVAL) == "invalid argument" and pk.strerror(0) == "ok"


def test_workspace_bytes_grows_with_context():
    cfg = pk.make_config(16, 32, 8, 64, 32, 8, 128)
    a, b = pk.proxykv_workspace_bytes(cfg, 8192, 8192), pk.proxykv_workspace_bytes(cfg, 32768, 32768)
    assert 0 < a < b < 8 << 30
    with pytest.raises(pk.ProxyKVError):
        pk.proxykv_workspace_bytes(cfg, 0, 10)


def test_argument_checks_run_before_any_device_call():
    lib = pk.load()
    ctx = pk.proxykv_create(pk.make_config(1, 4, 2, 64, 1, 4, 128))
    h = ctx.handle
    one = ctypes.c_void_p(16)      # never dereferenced: every case below fails validation first
    assert lib.proxykv_score(h, None, one, one, 0, 8, 8, 4, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_score(h, one, one, one, 0, 0, 8, 4, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_score(h, one, one, one, 0, 8, 8, 0, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_score(h, one, one, one, 5, 8, 8, 4, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_score(h, one, one, one, 0, 1 << 31, 8, 4, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_score(None, one, one, one, 0, 8, 8, 4, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_score_self(h, one, None, 0, 8, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_score_self(h, one, one, 0, 0, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_score_self(h, one, one, 7, 8, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_map(h, one, 8, None, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_map(h, one, 8, one, None) == pk.PROXYKV_ESTATE          # weights not set
    assert lib.proxykv_topk(h, one, 1, 8, 0, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_topk(h, one, 1, 8, 9, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_topk(h, one, 0, 8, 2, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_compact(h, one, one, one, 1, 8, 9, 128, one, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_compact(h, one, one, None, 1, 8, 2, 128, one, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_compact(h, one, one, one, 1, 8, 2, 100, one, one, None) == pk.PROXYKV_EUNSUPPORTED
    assert lib.proxykv_compact_inplace(h, one, one, one, 1, 8, 9, 128, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_compact_inplace(h, one, None, one, 1, 8, 2, 128, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_compact_inplace(h, one, one, one, 1, 8, 2, 1024, None) == pk.PROXYKV_EUNSUPPORTED
    assert lib.proxykv_mask(h, one, 1, 8, 0, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_mask(h, one, 1, 8, 2, None, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_topk_pooled(h, one, 1, 2, 8, 9, one, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_topk_pooled(h, one, 1, 2, 8, 2, one, None, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_topk_pooled(h, one, 1, 4096, 1 << 20, 2, one, one, None) == pk.PROXYKV_EINVAL   # heads * N too long
    assert lib.proxykv_compact_pooled(h, one, one, one, None, 1, 2, 8, 2, 128, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_compact_pooled(h, one, one, one, one, 1, 0, 8, 2, 128, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_compact_pooled(h, one, one, one, one, 1, 2, 8, 2, 1024, None) == pk.PROXYKV_EUNSUPPORTED
    K = ctypes.c_int64()
    assert lib.proxykv_prune(h, one, one, one, 0, 8, 8, 4, 0.0, one, one, one, one, one, None, None,
                             ctypes.byref(K), None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_prune(h, one, one, one, 0, 8, 8, 4, 0.5, one, one, one, one, one, None, None,
                             ctypes.byref(K), None) == pk.PROXYKV_ESTATE
    assert lib.proxykv_set_mapper_weights(h, one, 3) == pk.PROXYKV_EINVAL
    assert lib.proxykv_destroy(None) == pk.PROXYKV_OK
    pk.proxykv_destroy(ctx)


@pytest.mark.skipif(torch.cuda.is_available(), reason="only meaningful without a GPU")
def test_compute_calls_fail_loudly_without_a_gpu():
    ctx = pk.proxykv_create(pk.make_config(1, 4, 2, 64, 1, 4, 128))
    with pytest.raises(pk.ProxyKVError) as e:
        pk.proxykv_reserve(ctx, 64, 64)
    assert e.value.status == pk.PROXYKV_EHIP
    pk.proxykv_destroy(ctx)
