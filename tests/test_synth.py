"""The seeded input generator (CPU only): bit-exact against a numpy uint64
re-implementation, moments, determinism, planted structure."""
import numpy as np
import torch

from paper_2605_16360_amd import synth


def _np_irwin_hall(seed, tensor_id, start, count):
    M = np.uint64
    golden, m1, m2 = M(0x9E3779B97F4A7C15), M(0xBF58476D1CE4E5B9), M(0x94D049BB133111EB)
    with np.errstate(over="ignore"):
        key = M(synth.stream_key(seed, tensor_id))
        idx = np.arange(start, start + count, dtype=np.uint64)
        total = np.zeros(count, dtype=np.int64)
        for r in range(3):
            z = (idx * M(3) + M(r)) * golden + key
            z = z + golden
            z = (z ^ (z >> M(30))) * m1
            z = (z ^ (z >> M(27))) * m2
            z = z ^ (z >> M(31))
            for f in range(4):
                total += ((z >> M(16 * f)) & M(0xFFFF)).astype(np.int64)
    return ((total - 393210).astype(np.float32) / np.float32(65536.0))


def test_generator_matches_uint64_reference_and_is_counter_based():
    a = synth.irwin_hall(123, 7, 1000, 4096).numpy()
    np.testing.assert_array_equal(a, _np_irwin_hall(123, 7, 1000, 4096))
    whole = synth.normal_tensor((3, 5000), 123, 7, block=4096).numpy().ravel()
    np.testing.assert_array_equal(whole[1000:5096], a)
    assert not np.array_equal(synth.irwin_hall(123, 8, 1000, 4096).numpy(), a)


def test_generator_moments():
    x = synth.irwin_hall(synth.MASTER_SEED, 1, 0, 1 << 20).double()
    assert abs(float(x.mean())) < 5e-3 and abs(float(x.var()) - 1.0) < 1e-2
    assert float(x.abs().max()) <= 6.0 and float(x.abs().max()) > 3.5
    assert abs(float((x ** 4).mean()) - 2.9) < 0.05       # Irwin-Hall(12) kurtosis 3 - 0.1


def test_proxy_inputs_structure():
    c = synth.scaled_case(synth.CASES["llama_32k"], L_s=2, H_q=4, H_kv=2, N=1024, N_q=256, chunk=128,
                          n_planted=5, recency_band=64)
    q, kc, kr = synth.make_proxy_qk(c)
    q2, kc2, kr2 = synth.make_proxy_qk(c)
    assert q.dtype == torch.bfloat16 and torch.equal(q.view(torch.int16), q2.view(torch.int16))
    assert torch.equal(kc.view(torch.int16), kc2.view(torch.int16))
    assert q.shape == (2, 4, 256, 64) and kc.shape == (2, 2, 1024, 64) and kr.shape == (2, 2, 256, 64)
    plan = synth.plant_plan(c)
    for l in range(2):
        for h in range(2):
            assert len(set(plan["pos"][l, h].tolist())) == 5
            for p, g, i in zip(plan["pos"][l, h], plan["g"][l, h], plan["i"][l, h]):
                want = (3.0 * q[l, h * 2 + g, i].float()).to(torch.bfloat16)
                assert torch.equal(kc[l, h, p].view(torch.int16), want.view(torch.int16))
    # recency band: the mean of q.u is shifted by 0.5 d
    u = torch.from_numpy(plan["u"])
    proj = (q.float() * u.repeat_interleave(2, dim=1)[:, :, None, :]).sum(-1).mean()
    assert abs(float(proj) - 0.5 * 64) < 1.0
    t = synth.CASES["tiny"]
    qt, kt, _ = synth.make_proxy_qk(t)
    assert qt.dtype == torch.float32 and kt.dtype == torch.float32
    k_t, v_t = synth.make_target_kv(t)
    assert k_t.shape == (1, 4, 512, 128) and k_t.dtype == torch.bfloat16 and not torch.equal(k_t, v_t)


def test_mapper_weights_are_seeded_and_shaped():
    a = synth.make_mapper_weights(8, 8)
    b = synth.make_mapper_weights(8, 8)
    assert all(torch.equal(a[k], b[k]) for k in a) and list(a) == list(b)
    assert a["stem.conv1.weight"].shape == (256, 8, 3) and a["stem.conv2.weight"].shape == (512, 256, 3)
    assert a["enc.5.in_proj.weight"].shape == (1536, 512) and a["enc.0.ffn1.weight"].shape == (2048, 512)
    assert a["head.k_proj.weight"].shape == (512, 512) and a["head.queries"].shape == (8, 64)
    assert float(a["stem.bn1.var"].min()) >= 0.5
