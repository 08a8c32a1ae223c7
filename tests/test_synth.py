"""The seeded input generator: shapes, determinism and the stated distributions."""
import numpy as np
import torch

from oracle import lagkv_oracle as O
from paper_2504_04704_amd import synth


def test_config_table_matches_workloads():
    c = synth.CONFIGS
    assert c["cfg1_tiny_f32"].streams == 2
    assert c["cfg2_llama8b_16k"].streams == 256
    assert c["cfg4_llama8b_128k_b4"].streams == 1024
    assert c["cfg5_decode_b32"].streams == 8192
    for cfg in c.values():
        assert cfg.S == 16 and O.keep_count(cfg.L, cfg.r) in (32, 64, 128)


def test_make_kv_is_seeded_and_shaped():
    cfg = synth.CONFIGS["cfg2_llama8b_16k"].scaled(layers=2, T=512)
    K1, V1 = synth.make_kv(cfg)
    K2, V2 = synth.make_kv(cfg)
    assert K1.shape == (2, 8, 512, 128) and K1.dtype == torch.bfloat16
    assert torch.equal(K1, K2) and torch.equal(V1, V2)
    K3, _ = synth.make_kv(cfg, seed=7)
    assert not torch.equal(K1, K3)


def test_distributions():
    cfg = synth.CONFIGS["cfg2_llama8b_16k"].scaled(layers=1, T=4096)
    K, V = synth.make_kv(cfg)
    K = K.float(); V = V.float()
    oc = synth.outlier_channels(cfg, synth.MASTER_SEED, 0)
    assert oc.shape == (8, 4)
    ch_std = K[0].std(dim=1)                                   # [H, D]
    sK = synth.key_channel_scale(cfg, synth.MASTER_SEED, 0, "cpu")
    assert torch.allclose(ch_std, sK, rtol=0.08)
    base = torch.exp(torch.tensor(0.0))
    # outlier channels are an order of magnitude above the log-normal bulk
    med = ch_std.median(dim=1).values
    assert (ch_std.gather(1, oc) / med[:, None]).min() > 2.5
    tok_std = V[0].std(dim=2)                                  # [H, T]
    ls = torch.log(tok_std)
    assert abs(float(ls.mean())) < 0.05 and abs(float(ls.std()) - 0.3) < 0.06


def test_outlier_positions_per_layer_only_when_asked():
    c2 = synth.CONFIGS["cfg2_llama8b_16k"]; c3 = synth.CONFIGS["cfg3_llama8b_64k"]
    assert torch.equal(synth.outlier_channels(c2, 1, 0), synth.outlier_channels(c2, 1, 5))
    assert not torch.equal(synth.outlier_channels(c3, 1, 0), synth.outlier_channels(c3, 1, 5))


def test_oracle_on_config1():
    cfg = synth.CONFIGS["cfg1_tiny_f32"]
    K, V = synth.make_kv(cfg)
    for h in range(cfg.H):
        k, v = K[0, h].double().numpy(), V[0, h].double().numpy()
        Ko, Vo, idx, sc = O.compress(k, v, cfg.S, cfg.L, cfg.r)
        assert idx.shape[0] == 640 and sc.shape[0] == 6 * 128
        assert np.allclose(sc.reshape(6, 128).sum(axis=1), 2.0)


def test_stream_sample():
    s = synth.stream_sample(1024, 32)
    assert len(s) == 32 and s[0] == 0 and s[-1] == 1023 and len(set(s)) == 32
    assert synth.stream_sample(4, 32) == [0, 1, 2, 3]
