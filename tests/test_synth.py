"""The seeded input recipe: determinism, shapes, dtype rounding, identity statistics."""
import numpy as np
import torch

from paper_2512_07090_amd import synth


def test_workload_table_matches_benchmark_definition():
    w = synth.WORKLOADS
    assert [(x.dtype, x.batch, x.n_q_heads, x.n_kv_heads, x.seq, x.head_dim) for x in w] == [
        ("f32", 1, 32, 32, 512, 128), ("bf16", 8, 32, 32, 4096, 128),
        ("bf16", 4, 40, 40, 4096, 128), ("bf16", 2, 32, 8, 8192, 128),
        ("bf16", 1, 32, 8, 32768, 128)]
    assert w[1].prune_ratios == (0.25, 0.5)
    assert [x.n_prototypes for x in w] == [64, 256, 256, 512, 512]


def test_deterministic_and_shaped():
    w = synth.scaled(synth.workload(3), batch=1, seq=256)
    q1, k1, v1, z1 = synth.make_qkv(w)
    q2, k2, v2, z2 = synth.make_qkv(w)
    assert torch.equal(q1, q2) and torch.equal(k1, k2) and torch.equal(v1, v2) and torch.equal(z1, z2)
    assert q1.shape == (1, 32, 256, 128) and k1.shape == v1.shape == (1, 8, 256, 128)
    assert q1.dtype == torch.bfloat16 and q1.is_contiguous()


def test_repeated_identity_is_redundant_in_every_head():
    w = synth.scaled(synth.workload(0), seq=128)
    _, k, _, z = synth.make_qkv(w)
    zz = z[0]
    t0 = int(torch.nonzero(zz == zz.mode().values)[0])
    t1 = int(torch.nonzero(zz == zz.mode().values)[1])
    cos = torch.nn.functional.cosine_similarity(k[0, :, t0], k[0, :, t1], dim=-1)
    assert torch.all(cos > 0.8)            # same prototype + sigma 0.3 noise, in all 32 heads


def test_zipf_and_runs_statistics():
    gen = torch.Generator().manual_seed(1)
    w = synth.scaled(synth.workload(1), batch=2, seq=20000)
    z = synth.token_identities(w, gen)
    counts = torch.bincount(z.flatten(), minlength=w.n_prototypes).double()
    assert counts[0] > counts[1] > counts[3] > counts[15] > counts[100]
    ratio = counts[0] / counts[1]
    assert 2.0 < ratio < 2.6               # 2^1.2 = 2.30
    w5 = synth.scaled(synth.workload(4), seq=40000)
    z5 = synth.token_identities(w5, torch.Generator().manual_seed(2))[0].numpy()
    change = np.nonzero(np.diff(z5))[0]
    run_len = np.diff(change)
    assert run_len.max() <= 2 * 64         # adjacent runs may share an identity
    assert 6.0 < run_len.mean() < 10.5


def test_split_noise_heads():
    w = synth.scaled(synth.workload(2), batch=1, seq=64)
    _, k, _, z = synth.make_qkv(w)
    # spread of the per-head noise: low-noise heads sit closer to their prototypes
    lo = k[0, :20].float().std().item()
    hi = k[0, 20:].float().std().item()
    assert hi > 1.2 * lo
