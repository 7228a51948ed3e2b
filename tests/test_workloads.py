"""The seeded input generators: deterministic, rounded to the storage type, right structure."""
import numpy as np
import torch

from paper_2502_02406_amd import workloads as W


def tiny(**kw):
    d = dict(name="t", B=2, Hq=4, Hkv=2, D=64, Sq=40, Skv=300, dtype="bf16", std=0.5)
    d.update(kw)
    return W.Workload(**d)


def test_deterministic_and_seed_sensitive():
    a, b, c = W.make_inputs(tiny()), W.make_inputs(tiny()), W.make_inputs(tiny(), seed=7)
    for n in ("q", "k", "v", "do"):
        assert torch.equal(a[n], b[n])
        assert not torch.equal(a[n], c[n])
        assert a[n].dtype == torch.bfloat16
    assert a["q"].shape == (2, 4, 40, 64) and a["k"].shape == (2, 2, 300, 64)
    assert not torch.equal(a["q"].float()[:, :, :, :], a["do"].float())


def test_distribution_and_exact_widening():
    x = W.make_inputs(tiny(Sq=512, Skv=4096))
    k = W.as_f32_numpy(x["k"])
    assert abs(k.std() - 0.5) < 0.01 and abs(k.mean()) < 0.01
    assert np.array_equal(torch.from_numpy(k).to(torch.bfloat16).float().numpy(), k)   # bf16-exact


def test_outlier_rows():
    w = tiny(Skv=2000, outlier_frac=0.01, outlier_scale=8.0)
    tok = W.outlier_tokens(w)
    assert tok.shape == (2, 20) and len(set(tok[0])) == 20
    a = W.as_f32_numpy(W.make_inputs(w)["k"])
    b = W.as_f32_numpy(W.make_inputs(tiny(Skv=2000))["k"])
    for bi in range(2):
        hit = np.zeros(2000, bool); hit[tok[bi]] = True
        assert np.array_equal(a[bi][:, ~hit], b[bi][:, ~hit])
        ratio = np.abs(a[bi][:, hit]).mean() / np.abs(b[bi][:, hit]).mean()
        assert 7.5 < ratio < 8.5


def test_block_causal_mask_and_flop_counts():
    w = W.WORKLOADS["c4_flamingo_masked"]
    allow = W.block_causal_mask(w)
    assert allow.shape == (32, 128) and allow.sum() == 528
    assert allow[0, 0] == 1 and allow[0, 1] == 0 and allow[31, 31] == 1 and allow[31, 32] == 0
    assert abs(w.visible_pairs() / (w.Sq * w.Skv) - 528 / 4096) < 1e-12
    c3 = W.WORKLOADS["c3_longvideo_256k"]
    assert abs(c3.fwd_flops() - 8.796e12) < 1e9 and abs(c3.bwd_flops() - 21.99e12) < 1e10
    assert c3.Skv // c3.n_blocks == 32768
    c1 = W.WORKLOADS["c1_tiny"]
    assert c1.dtype == "f32" and W.make_inputs(c1)["q"].dtype == torch.float32


def test_recent_frame_mask_and_model_shaped_workloads():
    w = W.WORKLOADS["m3_flamingo_recent_frame"]
    allow = W.media_mask(w)
    assert allow.shape == (2048, 2048) and np.array_equal(allow, np.eye(2048, dtype=np.uint8))
    assert w.visible_pairs() == w.Sq * 64                      # every text row sees one frame of 64 tokens
    # more text chunks than frames: the late chunks keep the last frame
    late = W.scaled(w, Sq=16, Skv=3 * 64)
    assert np.array_equal(W.media_mask(late).argmax(axis=1), [0, 1, 2, 2, 2, 2, 2, 2])
    # ragged last chunk and block are counted by the rows and keys that exist
    rag = W.scaled(w, Sq=5, Skv=100, mask_kind="causal")       # chunks of 2,2,1 rows; blocks of 64, 36 keys
    assert rag.visible_pairs() == 2 * 64 + 2 * 100 + 1 * 100
    m1 = W.WORKLOADS["m1_owl7b_729"]
    assert m1.Skv == 2000 * 729 and m1.Skv % m1.n_blocks == 0 and (m1.Skv // m1.n_blocks) % 729 == 0
    m2 = W.WORKLOADS["m2_flamingo9b_64"]
    assert m2.Skv == 32768 * 64 and m2.Sq * 16 == 65536
    assert W.WORKLOADS["x5_d96_skv256k"].D == 96
