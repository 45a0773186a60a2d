"""GPU parity of the ragged / streaming entry points against the CPU oracle:
ragged selection and compaction into the slot cache, token append, ragged
decode attention and eviction to a budget, step by step.  Token-id sets, rows,
norm bits and lengths must match exactly; attention within 1e-4."""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_11430_amd as l2kv
from paper_2406_11430_amd import synth

pytestmark = pytest.mark.gpu
ATTN_BAR = 1e-4


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.fail("no HIP device visible: the gpu tests need a real MI355X")
    l2kv.lib()
    return torch.device("cuda:0")


def rows(rng, shape, dt, ties=False):
    x = rng.standard_normal(shape).astype(np.float32)
    x *= np.exp(0.5 * rng.standard_normal(shape[:-1] + (1,))).astype(np.float32)
    if ties:
        x[..., ::5, :] = x[..., :1, :]
    t = torch.from_numpy(x)
    return t.to(torch.bfloat16) if dt == "bf16" else t


def offsets(vals):
    return np.concatenate([[0], np.cumsum(vals)]).astype(np.int64)


class Batch:
    """A ragged batch on both sides: device tensors driven through the library and
    one oracle StreamHead per (plane, sequence)."""

    def __init__(self, dev, rng, dt, D, L, Hkv, G, lens, r, steps, ties=False, budget_fn=None):
        self.dev, self.dt, self.D, self.L, self.Hkv, self.G, self.r = dev, dt, D, L, Hkv, G, r
        self.lens0 = list(lens)
        self.n_seq, self.P = len(lens), L * Hkv
        self.budget_fn = budget_fn or (lambda seen, s: oracle.keep_count(seen, r))
        self.in_off = offsets(lens)
        ks = [min(n, self.budget_fn(n, s)) if n > 0 else 0 for s, n in enumerate(lens)]   # prompt compressed to its budget
        self.out_off = offsets(ks)
        # room for the largest budget of any step plus the token appended before the eviction
        # (an empty prompt grows like any other sequence: budget 0 before its first token)
        caps = [max(self.budget_fn(n + t, s) if n + t > 0 else 0 for t in range(steps + 1)) + 1
                for s, n in enumerate(lens)]
        self.slot_off = offsets(caps)
        total, total_kept, total_slots = int(self.in_off[-1]), int(self.out_off[-1]), int(self.slot_off[-1])
        K = rows(rng, (self.P, total, D), dt, ties)
        V = rows(rng, (self.P, total, D), dt)
        self.Kn, self.Vn = synth.as_numpy_bits(K), synth.as_numpy_bits(V)
        Kd, Vd = K.to(dev), V.to(dev)
        d_in, d_out, d_slot = (torch.from_numpy(a).to(dev) for a in (self.in_off, self.out_off, self.slot_off))
        self.d_slot = d_slot

        # ---- prompt compression on the device
        norms = torch.empty((self.P, total), dtype=torch.float32, device=dev)
        l2kv.l2kv_norms(Kd, norms)
        idx = torch.full((self.P, total_kept), -1, dtype=torch.int32, device=dev)
        l2kv.l2kv_select_ragged(norms, d_in, d_out, max(lens), idx)
        tdt = Kd.dtype
        self.Kc = torch.zeros((self.P, total_slots, D), dtype=tdt, device=dev)
        self.Vc = torch.zeros_like(self.Kc)
        self.nc = torch.zeros((self.P, total_slots), dtype=torch.float32, device=dev)
        self.pc = torch.full((self.P, total_slots), -1, dtype=torch.int32, device=dev)
        l2kv.l2kv_compact_ragged(Kd, Vd, norms, idx, d_in, d_out, max(ks), d_slot, self.Kc, self.Vc, self.nc, self.pc)
        self.lensA = torch.tensor(ks, dtype=torch.int32, device=dev)
        self.lensB = torch.zeros_like(self.lensA)
        self.idx_host = idx.cpu().numpy()
        self.norms_host = norms.cpu().numpy()

        # ---- the same on the oracle, head by head
        self.heads = {}
        for p in range(self.P):
            for s, n in enumerate(lens):
                h = oracle.StreamHead(caps[s], D, dt)
                if n > 0:
                    a, b = self.in_off[s], self.in_off[s + 1]
                    n32, _ = oracle.norms(self.Kn[p:p + 1, a:b], dt)
                    assert np.array_equal(self.norms_host[p, a:b].view(np.uint32), n32[0].view(np.uint32))
                    kept = oracle.select(n32, ks[s])[0]
                    assert np.array_equal(self.idx_host[p, self.out_off[s]:self.out_off[s + 1]], kept), (p, s)
                    h.load(self.Kn[p, a:b][kept], self.Vn[p, a:b][kept], n32[0, kept], kept.astype(np.int32))
                self.heads[(p, s)] = h
        self.check_cache(ks)

    def check_cache(self, want_lens):
        lens = self.lensA.cpu().numpy()
        assert list(lens) == list(want_lens)
        Kc, Vc = synth.as_numpy_bits(self.Kc), synth.as_numpy_bits(self.Vc)
        nc, pc = self.nc.cpu().numpy(), self.pc.cpu().numpy()
        for (p, s), h in self.heads.items():
            n, a = len(h), self.slot_off[s]
            assert n == lens[s], (p, s, n, lens[s])
            ids, Kk, Vk, nk = h.kept()
            order = np.argsort(pc[p, a:a + n], kind="stable")
            assert np.array_equal(pc[p, a:a + n][order], ids), (p, s)            # same token-id set
            assert np.array_equal(Kc[p, a:a + n][order], Kk) and np.array_equal(Vc[p, a:a + n][order], Vk)
            assert np.array_equal(nc[p, a:a + n][order].view(np.uint32), nk.view(np.uint32))

    def step(self, rng, t, n_splits=0, ordered=False):
        dev, D, L, Hkv, G = self.dev, self.D, self.L, self.Hkv, self.G
        Kn = rows(rng, (L, self.n_seq, Hkv, D), self.dt)
        Vn = rows(rng, (L, self.n_seq, Hkv, D), self.dt)
        tok = torch.tensor([n + t for n in self.lens0], dtype=torch.int32, device=dev)
        l2kv.l2kv_stream_append(Kn.to(dev), Vn.to(dev), tok, self.d_slot, self.lensA, self.lensB,
                                self.Kc, self.Vc, self.nc, self.pc)
        Knn, Vnn = synth.as_numpy_bits(Kn), synth.as_numpy_bits(Vn)
        for (p, s), h in self.heads.items():
            h.append(Knn[p // Hkv, s, p % Hkv], Vnn[p // Hkv, s, p % Hkv], self.lens0[s] + t)
        lens_now = self.lensB.cpu().numpy()
        assert list(lens_now) == [len(self.heads[(0, s)]) for s in range(self.n_seq)]

        # ---- attention, one layer at a time
        max_len = int(lens_now.max())
        Hq = Hkv * G
        ws = torch.zeros(l2kv.l2kv_decode_ragged_workspace_bytes(self.n_seq, Hq, max_len, D),
                         dtype=torch.uint8, device=dev)
        worst = 0.0
        order = None
        if ordered:
            order = torch.empty_like(self.lensB)
            l2kv.l2kv_length_order(self.lensB, order)
            assert np.array_equal(order.cpu().numpy(), oracle.length_order(lens_now))
        for layer in range(L):
            Q = rows(rng, (self.n_seq, Hq, D), self.dt)
            O = torch.full((self.n_seq, Hq, D), float("nan"), dtype=torch.float32, device=dev)
            l2kv.l2kv_decode_attn_ragged(Q.to(dev), self.Kc[layer * Hkv:(layer + 1) * Hkv],
                                         self.Vc[layer * Hkv:(layer + 1) * Hkv], self.lensB, self.d_slot,
                                         max_len, O, ws, n_splits=min(n_splits, l2kv.l2kv_decode_max_splits(max_len)),
                                         seq_order=order)
            got = O.cpu().numpy()
            Qn = synth.as_numpy_bits(Q)
            for s in range(self.n_seq):
                for hk in range(Hkv):
                    want = self.heads[(layer * Hkv + hk, s)].attend(Qn[s, hk * G:(hk + 1) * G])
                    worst = max(worst, float(np.abs(got[s, hk * G:(hk + 1) * G] - want).max()))
        assert worst <= ATTN_BAR, worst

        # ---- evict to the budget of the tokens seen so far
        budgets = [self.budget_fn(n + t + 1, s) for s, n in enumerate(self.lens0)]
        l2kv.l2kv_stream_evict(self.d_slot, self.lensB, torch.tensor(budgets, dtype=torch.int32, device=dev),
                               self.lensA, self.Kc, self.Vc, self.nc, self.pc)
        for (p, s), h in self.heads.items():
            h.evict_to(budgets[s])
        self.check_cache([min(int(lens_now[s]), budgets[s]) for s in range(self.n_seq)])


@pytest.mark.parametrize("dt,D", [("bf16", 128), ("f32", 64), ("bf16", 256)])
def test_stream_growing_budget(dev, dt, D):
    rng = np.random.default_rng(11 + D)
    b = Batch(dev, rng, dt, D, L=2, Hkv=2, G=2, lens=[70, 1, 333, 64, 129], r=0.5, steps=12)
    for t in range(12):
        b.step(rng, t)


def test_stream_sequences_that_start_empty(dev):
    # empty prompts in a batch: nothing to select or compact for them, then they grow token by
    # token like the others (append, attend over 1, 2, ... rows, evict to the growing budget)
    rng = np.random.default_rng(40)
    b = Batch(dev, rng, "bf16", 128, L=1, Hkv=2, G=4, lens=[0, 37, 0, 5], r=0.5, steps=7)
    for t in range(7):
        b.step(rng, t, n_splits=t % 2, ordered=bool(t % 2))


def test_stream_fixed_budget_with_ties_equals_one_shot_select(dev):
    # fixed budget: the kept set after every step must be the one-shot selection over all tokens
    # seen (the oracle pin); rows repeat so many norms tie and the token id decides
    rng = np.random.default_rng(5)
    lens = [40, 200, 17]
    fixed = [24, 90, 17]
    b = Batch(dev, rng, "bf16", 128, L=1, Hkv=3, G=4, lens=lens, r=0.5, steps=10, ties=True,
              budget_fn=lambda seen, s: fixed[s])
    for t in range(10):
        b.step(rng, t, n_splits=(t % 3))


def test_stream_budget_drop_evicts_several(dev):
    # the budget falls by a lot in one step: the eviction loop runs many times per head
    rng = np.random.default_rng(8)
    lens = [100, 90]
    after_step = [60, 60, 13, 13, 1]                 # budget after decode step t, both sequences

    def budget(seen, s):
        t = seen - lens[s] - 1                       # decode step this budget applies to
        return after_step[t] if 0 <= t < len(after_step) else 60

    b = Batch(dev, rng, "bf16", 128, L=1, Hkv=2, G=1, lens=lens, r=0.5, steps=5, budget_fn=budget)
    for t in range(5):
        b.step(rng, t)


def test_ragged_decode_lengths_and_splits(dev):
    # decode alone: lengths from 0 (zero output row) to several row tiles, every split count
    rng = np.random.default_rng(3)
    lens = [0, 1, 15, 64, 65, 700, 2049]
    Hkv, G, D, dt = 2, 4, 128, "bf16"
    slot_off = offsets([max(n, 1) + 3 for n in lens])
    total = int(slot_off[-1])
    K, V = rows(rng, (Hkv, total, D), dt), rows(rng, (Hkv, total, D), dt)
    Q = rows(rng, (len(lens), Hkv * G, D), dt)
    Kn, Vn, Qn = synth.as_numpy_bits(K), synth.as_numpy_bits(V), synth.as_numpy_bits(Q)
    d_lens = torch.tensor(lens, dtype=torch.int32, device=dev)
    d_off = torch.from_numpy(slot_off).to(dev)
    smax = l2kv.l2kv_decode_max_splits(max(lens))
    ws = torch.zeros(l2kv.l2kv_decode_ragged_workspace_bytes(len(lens), Hkv * G, max(lens), D),
                     dtype=torch.uint8, device=dev)
    lpt = torch.empty_like(d_lens)
    l2kv.l2kv_length_order(d_lens, lpt)
    assert np.array_equal(lpt.cpu().numpy(), oracle.length_order(lens))
    shuffled = torch.from_numpy(rng.permutation(len(lens)).astype(np.int32)).to(dev)
    for ns, order in ((0, None), (1, None), (2, None), (5, None), (smax, None), (0, lpt), (1, lpt), (3, lpt),
                      (0, shuffled), (2, shuffled)):
        O = torch.full((len(lens), Hkv * G, D), float("nan"), dtype=torch.float32, device=dev)
        l2kv.l2kv_decode_attn_ragged(Q.to(dev), K.to(dev), V.to(dev), d_lens, d_off, max(lens), O, ws, n_splits=ns,
                                     seq_order=order)
        got = O.cpu().numpy()
        assert np.all(got[0] == 0)                                   # empty sequence
        for s, n in enumerate(lens):
            if n == 0:
                continue
            a = slot_off[s]
            want = oracle.decode_attn(Qn[s:s + 1], Kn[None, :, a:a + n], Vn[None, :, a:a + n], dt)[0]
            assert np.abs(got[s] - want).max() <= ATTN_BAR, (ns, s)


def ragged_case(dev, rng, lens, Hkv, G, D=128, dt="bf16"):
    slot_off = offsets([max(n, 1) + 2 for n in lens])
    total = int(slot_off[-1])
    K, V = rows(rng, (Hkv, total, D), dt), rows(rng, (Hkv, total, D), dt)
    Q = rows(rng, (len(lens), Hkv * G, D), dt)
    host = tuple(synth.as_numpy_bits(t) for t in (Q, K, V))
    d_lens = torch.tensor(lens, dtype=torch.int32, device=dev)
    d_off = torch.from_numpy(slot_off).to(dev)
    return host, (Q.to(dev), K.to(dev), V.to(dev)), d_lens, d_off, slot_off


def check_ragged(got, host, lens, slot_off, dt, tag):
    Qn, Kn, Vn = host
    for s, n in enumerate(lens):
        if n == 0:
            assert np.all(got[s] == 0), (tag, s)
            continue
        a = slot_off[s]
        want = oracle.decode_attn(Qn[s:s + 1], Kn[None, :, a:a + n], Vn[None, :, a:a + n], dt)[0]
        assert np.abs(got[s] - want).max() <= ATTN_BAR, (tag, s)


@pytest.mark.parametrize("G", [2, 8])
def test_ragged_decode_work_list_with_more_items_than_workgroups(dev, G):
    # ordered launches hand (sequence, KV head, share) items to one workgroup per compute unit from a
    # device-side list: 40 sequences x 8 KV heads, whole sequences (320 items), two shares (640) and
    # twelve shares (3840 items, the merge variant for more than 8 workgroups per head); short
    # sequences use fewer shares than launched, so many items are skipped.  Run twice on the same
    # workspace: the list must be left ready for the next call.
    rng = np.random.default_rng(77)
    lens = [int(x) for x in rng.integers(1, 3000, 40)]
    lens[3], lens[17] = 0, 2999
    Hkv = 8                      # G = 8: the variant that forms q.k on the matrix unit
    host, (Qd, Kd, Vd), d_lens, d_off, slot_off = ragged_case(dev, rng, lens, Hkv, G)
    ws = torch.zeros(l2kv.l2kv_decode_ragged_workspace_bytes(len(lens), Hkv * G, max(lens), 128),
                     dtype=torch.uint8, device=dev)
    lpt = torch.empty_like(d_lens)
    l2kv.l2kv_length_order(d_lens, lpt)
    for rep in range(2):
        for ns, order in ((0, lpt), (2, lpt), (12, lpt), (0, None), (12, None)):
            O = torch.full((len(lens), Hkv * G, 128), float("nan"), dtype=torch.float32, device=dev)
            l2kv.l2kv_decode_attn_ragged(Qd, Kd, Vd, d_lens, d_off, max(lens), O, ws, n_splits=ns, seq_order=order)
            check_ragged(O.cpu().numpy(), host, lens, slot_off, "bf16", (rep, ns, order is not None))


def test_ragged_decode_under_graph_capture(dev):
    # ragged decode with and without a stored order (the latter ranks the lengths inside the call) is
    # made of plain launches: captured after an eager warm-up, replayed on changed queries and lengths
    # with eager calls in between, every replay bit-identical to the eager result
    rng = np.random.default_rng(78)
    lens = [2500, 64, 1300, 2100, 7, 900]
    Hkv, G = 4, 4
    host, (Qd, Kd, Vd), d_lens, d_off, slot_off = ragged_case(dev, rng, lens, Hkv, G)
    ws = torch.zeros(l2kv.l2kv_decode_ragged_workspace_bytes(len(lens), Hkv * G, max(lens), 128),
                     dtype=torch.uint8, device=dev)
    order = torch.empty_like(d_lens)
    O1 = torch.empty((len(lens), Hkv * G, 128), dtype=torch.float32, device=dev)
    O2 = torch.empty_like(O1)

    def path():
        l2kv.l2kv_length_order(d_lens, order)
        l2kv.l2kv_decode_attn_ragged(Qd, Kd, Vd, d_lens, d_off, max(lens), O1, ws, seq_order=order)
        l2kv.l2kv_decode_attn_ragged(Qd, Kd, Vd, d_lens, d_off, max(lens), O2, ws)        # self-ordered

    path()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        path()
    for rep in range(3):
        Qd.copy_(rows(rng, tuple(Qd.shape), "bf16").to(dev))
        new_lens = [max(1, n - 11 * rep) for n in lens]
        d_lens.copy_(torch.tensor(new_lens, dtype=torch.int32))
        path()
        torch.cuda.synchronize()
        want1, want2 = O1.clone(), O2.clone()
        O1.fill_(float("nan")); O2.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O1.view(torch.int32), want1.view(torch.int32)), rep
        assert torch.equal(O2.view(torch.int32), want2.view(torch.int32)), rep
        host_now = (synth.as_numpy_bits(Qd), host[1], host[2])
        check_ragged(O1.cpu().numpy(), host_now, new_lens, slot_off, "bf16", ("graph", rep))


def test_inconsistent_device_arrays_stay_inside_the_described_tensors(dev):
    # Offsets and lengths live on the device and cannot be validated by the host; the kernels force
    # them into the tensors the call describes.  Every tensor here is allocated with one spare plane
    # of sentinel values behind the described one, so a miss would land there (and be seen) instead
    # of outside the allocation.
    rng = np.random.default_rng(21)
    D, P, n_seq, total = 128, 2, 4, 300
    SENT = 1024.0                                  # exact in bf16

    def padded(shape_tail, dtype, fill):
        t = torch.full((P + 1,) + shape_tail, fill, dtype=dtype, device=dev)
        return t, t[:P]

    Kc_all, Kc = padded((total, D), torch.bfloat16, SENT)
    Vc_all, Vc = padded((total, D), torch.bfloat16, SENT)
    nc_all, nc = padded((total,), torch.float32, SENT)
    pc_all, pc = padded((total,), torch.int32, 777)
    Kc[:] = rows(rng, (P, total, D), "bf16").to(dev)
    Vc[:] = rows(rng, (P, total, D), "bf16").to(dev)
    nc[:] = 1.0
    pc[:] = 0
    bad_off = torch.tensor([-50, 100, 10 ** 12, 250, 90], dtype=torch.int64, device=dev)    # not ascending, out of range
    lens = torch.tensor([500, -3, 40, 10 ** 6], dtype=torch.int32, device=dev)
    lens_out = torch.zeros_like(lens)

    # append: rows go to clamped slots or nowhere
    Kn, Vn = rows(rng, (1, n_seq, P, D), "bf16").to(dev), rows(rng, (1, n_seq, P, D), "bf16").to(dev)
    tok = torch.arange(n_seq, dtype=torch.int32, device=dev)
    l2kv.l2kv_stream_append(Kn, Vn, tok, bad_off, lens, lens_out, Kc, Vc, nc, pc)
    # evict: budgets far below / above the lengths
    budgets = torch.tensor([1, 5, -7, 3], dtype=torch.int32, device=dev)
    lens2 = torch.zeros_like(lens)
    l2kv.l2kv_stream_evict(bad_off, lens, budgets, lens2, Kc, Vc, nc, pc)
    # decode over the same arrays
    Q = rows(rng, (n_seq, P * 2, D), "bf16").to(dev)
    ws = torch.zeros(l2kv.l2kv_decode_ragged_workspace_bytes(n_seq, P * 2, total, D), dtype=torch.uint8, device=dev)
    O = torch.full((n_seq, P * 2, D), float("nan"), dtype=torch.float32, device=dev)
    l2kv.l2kv_decode_attn_ragged(Q, Kc, Vc, lens, bad_off, total, O, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(O).all()
    assert torch.all(O[2] == 0)                        # sequence 2: offsets 10^12 .. 250 clamp to an empty range
    for spare, val in ((Kc_all[P], SENT), (Vc_all[P], SENT), (nc_all[P], SENT), (pc_all[P], 777)):
        assert torch.all(spare.float() == val)         # nothing was written behind the described planes
    got = lens2.cpu().numpy()
    assert got[0] <= 1 and got[1] == 0 and got[2] == 0 and got[3] <= 3

    # ragged selection and compaction with broken input / output offsets and indices
    total_in, total_kept = 400, 200
    norms_all = torch.full((P + 1, total_in), 3.0, dtype=torch.float32, device=dev)
    norms = norms_all[:P]
    norms[:] = torch.from_numpy(rng.random((P, total_in)).astype(np.float32)).to(dev)
    idx_all = torch.full((P + 1, total_kept), -9, dtype=torch.int32, device=dev)
    idx = idx_all[:P]
    in_off = torch.tensor([0, 500, -20, 390, 10 ** 9], dtype=torch.int64, device=dev)
    out_off = torch.tensor([0, 120, 10 ** 9, 150, 199], dtype=torch.int64, device=dev)
    l2kv.l2kv_select_ragged(norms, in_off, out_off, total_in, idx)
    K = rows(rng, (P, total_in, D), "bf16").to(dev)
    V = rows(rng, (P, total_in, D), "bf16").to(dev)
    idx[:, ::3] = 10 ** 8                              # indices far outside any sequence
    l2kv.l2kv_compact_ragged(K, V, norms, idx, in_off, out_off, total_kept, bad_off, Kc, Vc, nc, pc)
    torch.cuda.synchronize()
    assert torch.all(idx_all[P] == -9)
    for spare, val in ((Kc_all[P], SENT), (Vc_all[P], SENT), (nc_all[P], SENT), (pc_all[P], 777)):
        assert torch.all(spare.float() == val)
    assert int(pc.min()) >= 0 and int(pc.max()) < total_in


@pytest.mark.parametrize("n_seq", [1, 5, 64, 65, 257, 1500, 9000])
def test_length_order_exact(dev, n_seq):
    rng = np.random.default_rng(n_seq)
    lens = rng.integers(0, max(2, n_seq // 3), n_seq).astype(np.int32)          # many equal lengths
    order = torch.full((n_seq,), -1, dtype=torch.int32, device=dev)
    l2kv.l2kv_length_order(torch.from_numpy(lens).to(dev), order)
    assert np.array_equal(order.cpu().numpy(), oracle.length_order(lens))


def test_stream_random_batches(dev):
    # seeded random ragged batches (lengths, heads, group size, ratio, steps, split counts, with and
    # without a launch order) driven step by step against the oracle
    rng = np.random.default_rng(2406)
    for case in range(6):
        dt, D = (("bf16", 128), ("f32", 64), ("bf16", 64))[case % 3]
        n_seq = int(rng.integers(1, 7))
        lens = [int(x) for x in rng.integers(1, 400, n_seq)]
        steps = int(rng.integers(2, 7))
        b = Batch(dev, rng, dt, D, L=int(rng.integers(1, 3)), Hkv=int(rng.integers(1, 4)), G=int(rng.integers(1, 5)),
                  lens=lens, r=float(rng.uniform(0.1, 0.9)), steps=steps, ties=bool(case % 2))
        for t in range(steps):
            b.step(rng, t, n_splits=int(rng.integers(0, 3)), ordered=bool((case + t) % 2))
