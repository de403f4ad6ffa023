"""GPU parity outside the comfortable input regime, element by element against the float64
oracle through the C ABI (tolerances as everywhere: max abs 1e-2, relative L2 5e-3):

* every byte of the HBM arena (staging region included) and of the pinned host arena holds a
  NaN / Inf bit pattern before the KV is written, so the slots past a request's length, the
  unused blocks of its reservation and the staging copies' tails are poison, not zeros;
* non-default softmax scales and scaled queries (scores up to |s| ~ 1e3: one-hot weights,
  rescale factors that underflow);
* keys whose score rises along the sequence, so the running maximum moves on every tile;
* head groups of 1, 4, 8 and 16 query heads per KV head.

All of these are ordinary, valid inputs.
"""
import numpy as np
import pytest
import torch

from workloads import gen_kv, gen_q, gen_rising_k

pytestmark = pytest.mark.gpu

MAX_ABS, REL_L2, REL_L2_F32 = 1e-2, 5e-3, 3e-3
EDGE_LENS = [1, 17, 33, 1000, 1025]
POISON = {"quiet_nan": 0x7FC0, "plus_inf": 0x7F80, "all_ones": 0xFFFF}
DEV = "cuda:0"


class Case:
    """A liborbit context and the oracle's store holding the same explicit K/V tensors."""

    def __init__(self, kv, *, n_layers, Hq, Hkv, placement, scale=0.0, zero_copy=False, poison=None,
                 window=1, chunk=0, seed=0):
        from paper_2601_10729_amd import OrbitContext, orbit_plan_check
        from oracle import reference as ref
        self.ref, self.scale = ref, scale
        self.L, self.Hq, self.Hkv, self.D = n_layers, Hq, Hkv, 128
        self.lens = np.asarray([kv[(r, 0)][0].shape[0] for r in range(len(placement))], dtype=np.int32)
        self.ids = np.arange(len(self.lens), dtype=np.int64) + 50
        placement = np.asarray(placement, dtype=np.uint8)
        page_bytes = 2 * Hkv * 16 * 128 * 2
        _, _, need, _ = orbit_plan_check(self.lens, placement, 16, 0 if zero_copy else 1, window)
        blocks = int((-(-(self.lens.astype(np.int64) + window) // 16)).sum())
        self.hbm = torch.empty((need + 3) * page_bytes // 2, dtype=torch.int16, device=DEV)
        self.host = torch.empty((blocks * n_layers + 2) * page_bytes // 2, dtype=torch.int16, pin_memory=True)
        if poison is not None:
            bits = poison - 65536 if poison >= 32768 else poison
            self.hbm.fill_(bits)
            self.host.fill_(bits)
        torch.cuda.synchronize()
        self.cs, self.xs = torch.cuda.Stream(device=DEV), torch.cuda.Stream(device=DEV)
        self.ctx = OrbitContext(n_layers=n_layers, n_q_heads=Hq, n_kv_heads=Hkv, max_requests=len(self.lens),
                                max_tokens_per_request=int(self.lens.max()) + window + 16, softmax_scale=scale,
                                chunk_tokens=chunk, decode_window=window, zero_copy=zero_copy,
                                hbm_arena=self.hbm, host_arena=self.host, compute_stream=self.cs, copy_stream=self.xs)
        self.ctx.plan_load(self.ids, self.lens, placement)
        self.store = ref.PagedStore(n_layers, Hkv, 128, 16, blocks * n_layers + 4, seed=seed + 3)
        for r, rid in enumerate(self.ids):
            self.store.add_request(int(rid))
            for l in range(n_layers):
                k, v = kv[(r, l)]
                self.ctx.kv_fill(int(rid), l, 0, k.to(DEV), v.to(DEV))
                torch.cuda.synchronize()
                self.store.write(int(rid), l, 0, k.cpu(), v.cpu())

    def check_attention(self, layer, q):
        """q: [B][Hq][D] bf16 (cpu)."""
        out = torch.empty((len(self.ids), self.Hq, 128), dtype=torch.bfloat16, device=DEV)
        out32 = torch.empty(out.shape, dtype=torch.float32, device=DEV)
        qd = q.to(DEV).contiguous()
        torch.cuda.synchronize()
        self.ctx.decode_attention(layer, qd, out, out32)
        self.cs.synchronize()
        want = self.ref.decode_attention(self.store, layer, [int(i) for i in self.ids], q.contiguous(), self.Hq,
                                         scale=self.scale)
        self._compare(out, out32, want, ("attention", layer))

    def check_step(self, q_all, k_new, v_new):
        """One orbit_step: q_all [L][B][Hq][D], k_new / v_new [L][B][Hkv][D] (cpu)."""
        out = torch.empty((self.L, len(self.ids), self.Hq, 128), dtype=torch.bfloat16, device=DEV)
        args = [t.to(DEV).contiguous() for t in (q_all, k_new, v_new)]
        torch.cuda.synchronize()
        self.ctx.step(*args, out)
        self.cs.synchronize()
        self.xs.synchronize()
        for r, rid in enumerate(self.ids):
            for l in range(self.L):
                self.store.write(int(rid), l, int(self.lens[r]), k_new[l, r:r + 1], v_new[l, r:r + 1])
        self.lens = self.lens + 1
        for l in range(self.L):
            want = self.ref.decode_attention(self.store, l, [int(i) for i in self.ids], q_all[l].contiguous(), self.Hq,
                                             scale=self.scale)
            self._compare(out[l], None, want, ("step", l))

    @staticmethod
    def _compare(out, out32, want, what):
        assert np.isfinite(want).all()
        for got, bound in ((out, REL_L2), (out32, REL_L2_F32)):
            if got is None:
                continue
            g = got.detach().to(torch.float64).cpu().numpy()
            assert np.isfinite(g).all(), (what, "non-finite output")
            d = g - want
            ma = float(np.abs(d).max())
            rl = float(np.sqrt((d * d).sum() / max((want * want).sum(), 1e-300)))
            assert ma <= MAX_ABS and rl <= bound, (what, ma, rl)

    def close(self):
        torch.cuda.synchronize()
        self.ctx.destroy()


def _seeded_kv(lens, n_layers, Hkv, seed):
    return {(r, l): gen_kv(seed, l, 50 + r, 0, int(n), Hkv, 128, "cpu") for r, n in enumerate(lens) for l in range(n_layers)}


def _seeded_q(n_req, layer, Hq, seed, step=0):
    return torch.stack([gen_q(seed, layer, 50 + r, step, Hq, 128, "cpu") for r in range(n_req)])


@pytest.mark.parametrize("zero_copy", [False, True])
@pytest.mark.parametrize("poison", sorted(POISON))
def test_poisoned_arenas_do_not_reach_the_output(poison, zero_copy):
    """Layer 0 resident, layer 1 offloaded (staged through the poisoned staging region, or read in
    place); attention on both, then one orbit_step whose appended token lands in a poisoned slot."""
    Hq, Hkv, L = 8, 2, 2
    kv = _seeded_kv(EDGE_LENS, L, Hkv, seed=3)
    c = Case(kv, n_layers=L, Hq=Hq, Hkv=Hkv, placement=[[1, 0]] * len(EDGE_LENS), poison=POISON[poison],
             zero_copy=zero_copy)
    for layer in range(L):
        c.check_attention(layer, _seeded_q(len(EDGE_LENS), layer, Hq, seed=3))
    q_all = torch.stack([_seeded_q(len(EDGE_LENS), l, Hq, seed=3, step=1) for l in range(L)])
    new = [[gen_kv(3, l, 50 + r, int(n), 1, Hkv, 128, "cpu") for r, n in enumerate(EDGE_LENS)] for l in range(L)]
    k_new = torch.stack([torch.cat([kv_[0] for kv_ in row]) for row in new])
    v_new = torch.stack([torch.cat([kv_[1] for kv_ in row]) for row in new])
    c.check_step(q_all, k_new, v_new)
    c.close()


@pytest.mark.parametrize("G", [1, 8, 16])
def test_poisoned_arenas_other_group_sizes(G):
    Hkv, L = 2, 2
    Hq = G * Hkv
    kv = _seeded_kv(EDGE_LENS, L, Hkv, seed=4)
    c = Case(kv, n_layers=L, Hq=Hq, Hkv=Hkv, placement=[[1, 0], [0, 1], [1, 0], [0, 1], [1, 0]], poison=POISON["quiet_nan"])
    for layer in range(L):
        c.check_attention(layer, _seeded_q(len(EDGE_LENS), layer, Hq, seed=4))
    q_all = torch.stack([_seeded_q(len(EDGE_LENS), l, Hq, seed=4, step=1) for l in range(L)])
    new = [[gen_kv(4, l, 50 + r, int(n), 1, Hkv, 128, "cpu") for r, n in enumerate(EDGE_LENS)] for l in range(L)]
    k_new = torch.stack([torch.cat([kv_[0] for kv_ in row]) for row in new])
    v_new = torch.stack([torch.cat([kv_[1] for kv_ in row]) for row in new])
    c.check_step(q_all, k_new, v_new)
    c.close()


@pytest.mark.parametrize("G", [1, 4, 8, 16])
@pytest.mark.parametrize("scale", [0.01, 0.5, 1.0])
def test_softmax_scale_and_peaked_scores(scale, G):
    """Scores from nearly flat (scale 0.01) to |s| ~ 1e3 (scale 1.0, queries x 32): the weights go
    from uniform to one-hot, and the factor that shrinks the running accumulator underflows."""
    Hkv = 2
    Hq = G * Hkv
    lens = [33, 1000, 1025, 3000]
    kv = _seeded_kv(lens, 1, Hkv, seed=5)
    c = Case(kv, n_layers=1, Hq=Hq, Hkv=Hkv, placement=[[1]] * len(lens), scale=scale, chunk=256)
    q = _seeded_q(len(lens), 0, Hq, seed=5)
    for mult in (1.0, 8.0, 32.0):
        c.check_attention(0, (q.float() * mult).to(torch.bfloat16))
    c.close()


def test_query_aligned_with_one_key_selects_its_value():
    """q = 24 * k_j at scale 1: the score of token j exceeds every other by hundreds, so the output
    must be v_j to within the output rounding (the one-hot limit, on the GPU)."""
    Hq, Hkv = 8, 2
    lens = [1025, 2000]
    kv = _seeded_kv(lens, 1, Hkv, seed=6)
    c = Case(kv, n_layers=1, Hq=Hq, Hkv=Hkv, placement=[[1]] * 2, scale=1.0, chunk=512)
    picks = [[5, 1024, 700, 31, 32, 1000, 0, 513], [1999, 16, 1023, 1024, 1025, 3, 100, 64]]
    q = torch.empty((2, Hq, 128), dtype=torch.bfloat16)
    for r in range(2):
        for h in range(Hq):
            q[r, h] = (kv[(r, 0)][0][picks[r][h], h // 4].float() * 24.0).to(torch.bfloat16)
    out = torch.empty((2, Hq, 128), dtype=torch.bfloat16, device=DEV)
    c.ctx.decode_attention(0, q.to(DEV), out)
    c.cs.synchronize()
    for r in range(2):
        for h in range(Hq):
            assert torch.equal(out[r, h].cpu(), kv[(r, 0)][1][picks[r][h], h // 4]), (r, h)
    c.check_attention(0, q)
    c.close()


@pytest.mark.parametrize("G", [1, 4, 8, 16])
def test_scores_rising_along_the_sequence(G):
    """The score grows with the token index, so every tile raises the running maximum and every
    earlier partial sum is rescaled; rises of 30 and 600 natural-log units over the sequence."""
    Hkv = 2
    Hq = G * Hkv
    lens = [17, 1000, 1025, 4100]
    for rise, scale in ((30.0, 1.0), (600.0, 1.0), (30.0 * 128 ** 0.5, 0.0)):
        kv, q = {}, torch.empty((len(lens), Hq, 128), dtype=torch.bfloat16)
        for r, n in enumerate(lens):
            k, qdir = gen_rising_k(7, 0, 50 + r, n, Hkv, 128, rise, "cpu")
            _, v = gen_kv(7, 0, 50 + r, 0, n, Hkv, 128, "cpu")
            kv[(r, 0)] = (k, v)
            q[r] = qdir.view(1, 128).expand(Hq, 128)
        c = Case(kv, n_layers=1, Hq=Hq, Hkv=Hkv, placement=[[1]] * len(lens), scale=scale, chunk=128)
        c.check_attention(0, q)
        c.close()
