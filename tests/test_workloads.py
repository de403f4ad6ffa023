"""The seeded input generators: integer hash agrees with a Python-int reference, the value
table is a bf16 standard normal, and the five workloads have the stated shapes."""
import numpy as np
import torch

from workloads import synth


def test_torch_hash_matches_python_ints():
    key = synth.stream_key(5, synth.TENSOR_V, 3, 1001)
    idx = torch.tensor([0, 1, 2, 12345, 2**31 + 7, 2**40 + 11], dtype=torch.int64)
    got = synth._draw(key, idx)
    table = synth.normal_bf16_table()
    for i, want_idx in enumerate(int(x) for x in idx):
        assert got[i].item() == table[synth.draw_int(key, want_idx)].item()


def test_table_is_a_bf16_standard_normal():
    t = synth.normal_bf16_table().to(torch.float64)
    assert torch.all(t[1:] >= t[:-1])
    assert abs(t.mean().item()) < 1e-6 and abs(t.std().item() - 1.0) < 2e-3
    assert t.abs().max().item() < 4.4
    assert torch.equal(t, -t.flip(0))


def test_values_are_slice_and_head_consistent():
    k, v = synth.gen_kv(1, 2, 77, 0, 40, 8, 128)
    k2, v2 = synth.gen_kv(1, 2, 77, 10, 5, 8, 128, heads=[3, 6], max_elems=1024)
    assert torch.equal(k[10:15, [3, 6]], k2) and torch.equal(v[10:15, [3, 6]], v2)
    kn, vn = synth.gen_kv_new(1, 2, 77, 39, 8, 128)
    assert torch.equal(kn, k[39]) and torch.equal(vn, v[39])
    assert not torch.equal(k, v)
    q = synth.gen_q(1, 2, 77, 0, 32, 128)
    assert q.shape == (32, 128) and q.dtype == torch.bfloat16
    assert abs(k.float().std().item() - 1.0) < 0.02


def test_workload_shapes():
    t = synth.make_workload("tiny")
    assert list(t.ctx_len) == [17, 256, 1000, 2048] and t.n_layers == 2
    assert t.placement[:, 0].all() and not t.placement[:, 1].any()
    assert t.kv_bytes_per_token_layer == 1024 and t.page_bytes == 16 * 1024
    w = synth.make_workload("llama8b_b16")
    assert w.n_req == 16 and w.ctx_len.min() >= 8192 and w.ctx_len.max() <= 32768
    assert (w.placement.sum(axis=1) == 24).all() and w.page_bytes == 64 * 1024
    lc = synth.make_workload("long_ctx")
    assert lc.n_req == 4 and (lc.placement.sum(axis=1) == 16).all() and lc.steps == 32
    assert lc.ctx_len.min() >= 65536 and lc.ctx_len.max() <= 131072
    hm = synth.make_workload("heavy_mixed")
    assert hm.n_req == 64 and hm.ctx_len.min() >= 1024 and hm.ctx_len.max() <= 65536
    b = hm.blocks(hm.steps)
    used = int((hm.placement * b[:, None]).sum()) + int(((1 - hm.placement) * b[:, None]).sum(axis=0).max())
    assert used * hm.page_bytes <= 40 * 10**9
    big = synth.make_workload("llama70b")
    assert big.n_layers == 80 and big.n_q_heads == 64 and (big.placement.sum(axis=1) == 20).all()
    assert (big.placement == big.placement[0]).all()
    assert synth.make_workload("llama8b_b16", seed=1).ctx_len.tolist() != w.ctx_len.tolist()
    assert synth.make_workload("llama8b_b16", n_req=4).n_req == 4


def test_pack_bitmap_is_lsb_first():
    pl = np.zeros((2, 10), dtype=np.uint8)
    pl[0, 0] = 1
    pl[0, 9] = 1
    pl[1, 3] = 1
    bm = synth.pack_bitmap(pl)
    assert bm.shape == (2, 2) and bm.tolist() == [[1, 2], [8, 0]]
