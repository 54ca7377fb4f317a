"""The seeded input generators: shapes, determinism, and the stated distributions."""
import math

import torch

from paper_2506_06266_amd import synth


def test_attn_inputs_shapes_and_determinism():
    cfg = synth.ATTN_CONFIGS["cfg1_attn"]
    a = synth.attn_inputs(cfg)
    b = synth.attn_inputs(cfg)
    assert a["q"].shape == (2, 64, 2, 64) and a["k_own"].shape == (2, 64, 1, 64)
    assert a["z_k"].shape == (1, 32, 64) and a["d_o"].dtype == torch.float32
    for k in a:
        assert torch.equal(a[k], b[k])
    assert abs(a["q"].std().item() - 1.0) < 0.05
    assert abs(a["z_k"].std().item() - 1.0 / 8.0) < 0.01


def test_kl_inputs_teacher_is_distinct_sorted_and_has_the_stated_mass():
    cfg = synth.KL_CONFIGS["cfg1_loss"]
    t = synth.kl_inputs(cfg)
    assert t["logits"].shape == (128, 1000) and t["teacher_idx"].dtype == torch.int32
    idx = t["teacher_idx"].long()
    assert idx.min() >= 0 and idx.max() < cfg.V
    s, _ = idx.sort(dim=1)
    assert (s[:, 1:] != s[:, :-1]).all()
    p = t["teacher_logp"].double().exp()
    assert (p.sum(dim=1) - cfg.mass).abs().max() < 1e-6
    assert (p[:, 1:] <= p[:, :-1]).all()
    assert abs(t["logits"].std().item() - 2.0) < 0.05


def test_decode_inputs_ragged_lengths():
    cfg = synth.DECODE_CONFIGS["decode_small"]
    t = synth.decode_inputs(cfg)
    cu = t["cu_lens"].long()
    lens = cu[1:] - cu[:-1]
    assert cu[0] == 0 and lens.min() >= cfg.min_len and lens.max() <= cfg.max_len
    assert t["k_own"].shape == (int(cu[-1]), cfg.Hkv, cfg.D)
    assert t["k_own"].dtype == torch.bfloat16
    assert abs(t["k_own"].float().std().item() - 1 / math.sqrt(128)) < 0.01


def test_packed_inputs_lengths_and_offsets():
    cfg = synth.PACKED_CONFIGS["ragged_packed"]
    lens = synth.packed_lengths(cfg)
    assert lens.numel() == cfg.n_seq and lens.min() >= cfg.min_len and lens.max() <= cfg.max_len
    t = synth.attn_packed_inputs(cfg)
    cu = t["cu_seqlens"]
    assert cu.dtype == torch.int32 and cu[0] == 0 and torch.equal((cu[1:] - cu[:-1]).long(), lens)
    T = int(lens.sum())
    assert t["q"].shape == (T, 8, 128) and t["k_own"].shape == (T, 2, 128) and t["z_k"].shape == (2, 333, 128)
    assert torch.equal(t["q"], synth.attn_packed_inputs(cfg)["q"])
    big = synth.packed_lengths(synth.PACKED_CONFIGS["cfg3_packed"])
    assert big.numel() == 64 and big.max() <= 1024 and 30000 < int(big.sum()) < 40000
