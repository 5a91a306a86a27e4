"""Kernel-level parity: each single-operation entry point against the CPU oracle."""
import numpy as np
import pytest

from oracle import sampling as osamp
from oracle import transformer as otf
from paper_2601_05475_amd import binding, synth

from gpu_common import ATT_REL, check_sampler_on_logits, rel_l2

pytestmark = pytest.mark.gpu


def to_dev(a, dtype):
    """numpy fp32 values -> device tensor of the model dtype; returns (tensor, values as fp32)."""
    import torch
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda(), np.asarray(a, np.float32)
    t = torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(torch.bfloat16)
    return t.cuda(), t.to(torch.float32).numpy()


def rnd(seed, shape, std=1.0):
    return synth.normal(seed, 9, shape, 0.0, std, "f32")


TOL = {"f32": 2e-5, "bf16": 1e-2}      # relative to the output scale; bf16 outputs are rounded


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_add_rmsnorm(dtype):
    import torch
    rows, d, S = 5, 300, 3
    x = rnd(1, (rows, d)); parts = rnd(2, (S, rows, d), 0.3); g = 1 + rnd(3, (d,), 0.1)
    gd, gv = to_dev(g, dtype)
    xd = torch.from_numpy(x.copy()).cuda(); pd = torch.from_numpy(parts).cuda()
    h = binding.op_add_rmsnorm(xd, pd, gd, 1e-6)
    xs = x.astype(np.float64) + parts.astype(np.float64).sum(0)
    np.testing.assert_allclose(xd.cpu().numpy(), xs, rtol=0, atol=1e-6)
    want = otf.rmsnorm(xs, gv, 1e-6)
    np.testing.assert_allclose(h.float().cpu().numpy(), want, rtol=0, atol=TOL[dtype] * 4)
    h0 = binding.op_add_rmsnorm(xd, None, gd, 1e-6)          # no partials: x untouched
    np.testing.assert_array_equal(h0.float().cpu().numpy(), h.float().cpu().numpy())


@pytest.mark.parametrize("dtype,M,N,K,S", [
    ("f32", 3, 70, 100, 1), ("f32", 3, 70, 100, 3), ("f32", 130, 65, 33, 1),
    ("bf16", 4, 96, 200, 2), ("bf16", 32, 256, 512, 4), ("bf16", 16, 3072, 2048, 1),
    ("bf16", 200, 128, 256, 1), ("bf16", 33, 130, 72, 1),
])
def test_linear(dtype, M, N, K, S):
    a = rnd(4, (M, K)); w = rnd(5, (N, K), 0.05)
    ad, av = to_dev(a, dtype); wd, wv = to_dev(w, dtype)
    print("case: linear", dtype, M, N, K, S, flush=True)
    out = binding.op_linear(ad, wd, S).cpu().numpy().astype(np.float64).sum(0)
    want = otf.linear(av, wv)
    np.testing.assert_allclose(out, want, rtol=0, atol=2e-5 * np.abs(want).max() + 1e-6)


@pytest.mark.parametrize("dtype,M,N,K", [("f32", 5, 70, 100), ("bf16", 4, 96, 200), ("bf16", 32, 512, 256),
                                         ("bf16", 150, 128, 128)])
def test_linear_swiglu(dtype, M, N, K):
    a = rnd(6, (M, K)); wg = rnd(7, (N, K), 0.2); wu = rnd(8, (N, K), 0.2)
    ad, av = to_dev(a, dtype); gd, gv = to_dev(wg, dtype); ud, uv = to_dev(wu, dtype)
    out = binding.op_linear_swiglu(ad, gd, ud).float().cpu().numpy()
    want = otf.silu(otf.linear(av, gv)) * otf.linear(av, uv)
    np.testing.assert_allclose(out, want, rtol=0, atol=TOL[dtype] * np.abs(want).max())


def make_pools(dtype, n_pages, Hkv, pg, hd, seed):
    """Random K / V page pools in the library's page layout; returns device tensors and fp32
    views k[page, kvh, j, :], v[page, kvh, j, :] for the oracle."""
    k = rnd(seed, (n_pages, Hkv, pg, hd)); v = rnd(seed + 1, (n_pages, Hkv, pg, hd))
    kd, kv = to_dev(k, dtype)
    vd, vv = to_dev(v, dtype)
    kp, vp = binding.kv_pages_pack(kd, vd)
    return kp, vp, kv, vv


@pytest.mark.parametrize("dtype,pg", [("f32", 8), ("bf16", 8), ("f32", 32), ("bf16", 64)])
def test_rope_kv_write(dtype, pg):
    import torch
    rows, Hq, Hkv, hd, S, base = 7, 4, 2, 64, 2, 10000.0
    nq = (Hq + 2 * Hkv) * hd
    qkv = rnd(10, (S, rows, nq))
    pos = np.array([0, 1, 5, 130, 4095, 17000, 3], np.int32)
    page = np.array([3, 0, 2, 2, 1, 4, 0], np.int32)
    off = np.array([0, 7, 1, 2, 5, 6, 3], np.int32)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    kp = torch.zeros((5, Hkv, pg * hd), dtype=tdt, device="cuda")
    vp = torch.zeros((5, Hkv, pg * hd), dtype=tdt, device="cuda")
    q = binding.op_rope_kv_write(torch.from_numpy(qkv).cuda(), torch.from_numpy(pos).cuda(),
                                 torch.from_numpy(page).cuda(), torch.from_numpy(off).cuda(),
                                 Hq, Hkv, hd, pg, base, kp, vp)
    full = qkv.astype(np.float64).sum(0).reshape(rows, Hq + 2 * Hkv, hd)
    wq = otf.rope(full[:, :Hq], pos, base)
    wk = otf.rope(full[:, Hq:Hq + Hkv], pos, base)
    wv = full[:, Hq + Hkv:]
    tol = 1e-5 if dtype == "f32" else 2e-2
    np.testing.assert_allclose(q.float().cpu().numpy(), wq, rtol=0, atol=tol)
    ku, vu = binding.kv_pages_unpack(kp, vp, pg, hd)
    kh, vh = ku.float().cpu().numpy(), vu.float().cpu().numpy()
    for r in range(rows):
        np.testing.assert_allclose(kh[page[r], :, off[r], :], wk[r], rtol=0, atol=tol)
        np.testing.assert_allclose(vh[page[r], :, off[r], :], wv[r], rtol=0, atol=tol)
    written = np.zeros((5, pg), bool); written[page, off] = True
    assert np.all(kh[~written[:, None, :, None].repeat(Hkv, 1).repeat(hd, 3)] == 0)


def plant_key(kv, vv, kd_pool, vd_pool, page, kvh, slot, q_row, gain, dtype):
    """Make key `slot` of (page, kvh) a multiple of q_row, so that it takes nearly all of that
    row's softmax weight; host views and device pools are updated alike."""
    import torch
    pg, hd = kv.shape[2], kv.shape[3]
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    kt = torch.from_numpy(np.ascontiguousarray(gain * q_row, np.float32)).to(tdt)
    kv[page, kvh, slot] = kt.to(torch.float32).numpy()
    k_off, _ = binding.kv_page_offsets(pg, hd)
    kd_pool[page, kvh, torch.from_numpy(k_off[slot]).cuda()] = kt.cuda()


def attention_case(dtype, B, Hq, Hkv, hd, pg, P, t, splits=0, seed=20, stride=1, qscale=1.0, plant=()):
    """Decode attention against the oracle.  plant: (b, a, where, pos) tuples: the key at prefix /
    suffix position pos of row (b, a)'s KV head becomes 3 q[b, a] (score ~ 3 sqrt(hd) + the rest
    ~ N(0, 1): that key alone decides the output).  Returns (worst relative L2 over the compared
    rows, out, relative errors of the planted rows)."""
    import torch
    n_pre = -(-P // pg) if P else 0
    per = -(-t // pg) if t else 0
    kpd, vpd, kpv, vpv = make_pools(dtype, max(n_pre, 1), Hkv, pg, hd, seed)
    ksd, vsd, ksv, vsv = make_pools(dtype, max(B * per, 1), Hkv, pg, hd, seed + 2)
    table = np.random.default_rng(seed).permutation(max(B * per, 1)).astype(np.int32).reshape(B, -1) if per else np.zeros((B, 1), np.int32)
    q = rnd(seed + 4, (B, Hq, hd), qscale)
    qd, qv = to_dev(q, dtype)
    G = Hq // Hkv
    for b, a, where, pos in plant:
        if where == "prefix":
            plant_key(kpv, vpv, kpd, vpd, pos // pg, a // G, pos % pg, qv[b, a], 3.0 / qscale, dtype)
        else:
            plant_key(ksv, vsv, ksd, vsd, table[b, pos // pg], a // G, pos % pg, qv[b, a], 3.0 / qscale, dtype)
    print("case: attention", dtype, B, Hq, Hkv, hd, pg, P, t, splits, plant, flush=True)
    out = binding.op_attention_decode(qd, kpd if P else None, vpd if P else None, ksd if t else None,
                                      vsd if t else None, torch.from_numpy(table).cuda() if t else None,
                                      P, t, pg, splits).float().cpu().numpy()

    def want_row(b, a):
        c = a // G
        keys = [kpv[:, c].reshape(-1, hd)[:P]] if P else []
        vals = [vpv[:, c].reshape(-1, hd)[:P]] if P else []
        if t:
            keys.append(ksv[table[b, :per], c].reshape(-1, hd)[:t])
            vals.append(vsv[table[b, :per], c].reshape(-1, hd)[:t])
        return otf.attention_one(qv[b, a], np.concatenate(keys), np.concatenate(vals))

    worst = 0.0
    for b in range(B):
        for a in range(Hq):
            if (b * Hq + a) % stride:
                continue
            worst = max(worst, rel_l2(out[b, a], want_row(b, a)))
    planted = [rel_l2(out[b, a], want_row(b, a)) for b, a, _, _ in plant]
    return worst, out, planted


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Hq,Hkv,hd,pg,P,t", [
    (4, 4, 2, 64, 4, 128, 16), (3, 8, 2, 128, 64, 300, 70), (2, 4, 4, 32, 8, 0, 9),
    (5, 6, 2, 64, 16, 77, 0), (1, 4, 1, 128, 64, 1, 1), (32, 32, 8, 128, 64, 1024, 130),
])
def test_attention_decode(dtype, B, Hq, Hkv, hd, pg, P, t):
    worst, _, _ = attention_case(dtype, B, Hq, Hkv, hd, pg, P, t)
    assert worst < ATT_REL[dtype], worst


@pytest.mark.parametrize("dtype,B,Hq,Hkv,hd,pg,P,t", [
    ("f32", 5, 4, 2, 64, 4, 30, 19), ("bf16", 6, 8, 2, 128, 64, 300, 200), ("bf16", 9, 32, 8, 128, 64, 1000, 333),
    ("bf16", 4, 8, 4, 64, 64, 0, 130), ("bf16", 3, 8, 2, 96, 64, 100, 70),
])
def test_attention_decode_candidates_of_different_lengths(dtype, B, Hq, Hkv, hd, pg, P, t):
    """row_len: every candidate attends to its own number of suffix keys (1 .. t; some end inside
    the first block, some on a block or page edge, one is at the maximum), against the oracle's
    attention on exactly those keys."""
    import torch
    n_pre = -(-P // pg) if P else 0
    per = -(-t // pg)
    kpd, vpd, kpv, vpv = make_pools(dtype, max(n_pre, 1), Hkv, pg, hd, 41)
    ksd, vsd, ksv, vsv = make_pools(dtype, B * per, Hkv, pg, hd, 43)
    rng = np.random.default_rng(44)
    table = rng.permutation(B * per).astype(np.int32).reshape(B, per)
    lens = rng.integers(1, t + 1, B).astype(np.int32)
    lens[0], lens[1] = t, 1
    if B > 2:
        lens[2] = min(t, 32)
    if B > 3:
        lens[3] = min(t, pg)
    q = rnd(45, (B, Hq, hd))
    qd, qv = to_dev(q, dtype)
    print("case: ragged attention", dtype, B, Hq, Hkv, hd, pg, P, t, lens.tolist(), flush=True)
    out = binding.op_attention_decode(qd, kpd if P else None, vpd if P else None, ksd, vsd,
                                      torch.from_numpy(table).cuda(), P, t, pg,
                                      row_len=torch.from_numpy(lens).cuda()).float().cpu().numpy()
    G = Hq // Hkv
    worst = 0.0
    for b in range(B):
        for a in range(Hq):
            c = a // G
            keys = [kpv[:, c].reshape(-1, hd)[:P]] if P else []
            vals = [vpv[:, c].reshape(-1, hd)[:P]] if P else []
            keys.append(ksv[table[b], c].reshape(-1, hd)[:lens[b]])
            vals.append(vsv[table[b], c].reshape(-1, hd)[:lens[b]])
            want = otf.attention_one(qv[b, a], np.concatenate(keys), np.concatenate(vals))
            worst = max(worst, rel_l2(out[b, a], want))
    assert worst < ATT_REL[dtype], worst


@pytest.mark.parametrize("B,Hq,Hkv,hd,P,t,stride", [
    (32, 32, 8, 128, 4096, 512, 7),      # 8B-shape headline workload at its last step
    (32, 32, 8, 128, 4096, 1, 7),        # ... and at its first
    (16, 32, 8, 64, 2048, 256, 5),       # 1B shape
    (64, 40, 8, 128, 16384, 1024, 41),   # 32B shape: 320 query rows per KV head, 3 row blocks
    (64, 32, 8, 128, 4096, 0, 13),       # reranking fan-out, prefix only
    (2, 8, 8, 128, 63, 65, 1), (3, 8, 4, 64, 65, 64, 1), (5, 16, 2, 128, 129, 127, 1),
    (1, 32, 1, 64, 128, 129, 1), (7, 4, 2, 128, 0, 200, 1), (33, 8, 2, 128, 257, 1, 1),
    # many query rows per KV head
    (50, 32, 8, 128, 1000, 70, 3),       # 7 row blocks (the last of 8 rows), last page of 40 keys
    (64, 32, 2, 64, 200, 33, 17),        # head_dim 64, 32 row blocks, last page of 8 keys
    (48, 16, 4, 128, 130, 5, 1),         # 6 row blocks, 3 pages (the last with 2 keys)
    (64, 32, 8, 128, 100, 0, 3),         # 8 row blocks, one key split, no suffix: every item writes its outputs itself
    (72, 32, 8, 128, 700, 40, 5),        # 9 row blocks: three items of 4, 4 and 1 row blocks per KV head and split
])
def test_attention_decode_mfma_shapes(B, Hq, Hkv, hd, P, t, stride):
    worst, _, _ = attention_case("bf16", B, Hq, Hkv, hd, 64, P, t, stride=stride)
    assert worst < ATT_REL["bf16"], worst


@pytest.mark.parametrize("B,Hq,Hkv,hd,P,t,plant", [
    # 8B headline shape at its last step: one key deep inside the last prefix split, one in the
    # last 32-key block of a candidate's last suffix page, one in a middle page
    (32, 32, 8, 128, 4096, 512, [(5, 9, "prefix", 4000), (31, 31, "suffix", 500), (17, 2, "suffix", 200), (0, 0, "prefix", 33)]),
    # 32B shape: 320 query rows per KV head, 128 blocks per... many prefix splits
    (64, 40, 8, 128, 16384, 1024, [(63, 39, "prefix", 16383), (40, 17, "prefix", 9000), (7, 3, "suffix", 1023), (22, 36, "suffix", 70)]),
    (16, 32, 8, 64, 2048, 256, [(15, 31, "prefix", 2047), (3, 4, "suffix", 255), (9, 20, "suffix", 64)]),       # 1B shape
    (64, 32, 8, 128, 4096, 0, [(63, 0, "prefix", 4095), (1, 30, "prefix", 2049)]),                                # prefix only
    (7, 4, 2, 128, 0, 200, [(6, 3, "suffix", 199), (0, 0, "suffix", 130)]),                                       # suffix only
])
def test_attention_decode_one_key_decides(B, Hq, Hkv, hd, P, t, plant):
    """A key far inside a late prefix split or a late suffix page carries nearly all the weight of
    one row: a kernel that dropped its block, its page or its split's partial state would be O(1)
    wrong there."""
    worst, _, planted = attention_case("bf16", B, Hq, Hkv, hd, 64, P, t, stride=37, plant=plant)
    assert max(planted) < ATT_REL["bf16"], planted
    assert worst < ATT_REL["bf16"], worst


def test_attention_split_count_invariance():
    plant = [(7, 31, "prefix", 2040), (2, 5, "prefix", 1000)]
    outs = [attention_case("bf16", 8, 32, 8, 128, 64, 2048, 100, splits=s, plant=plant) for s in (1, 2, 8, 32)]
    for worst, o, planted in outs:
        assert worst < ATT_REL["bf16"] and max(planted) < ATT_REL["bf16"], (worst, planted)
    for _, o, _ in outs[1:]:
        # different splits round differently, in the last bf16 bit of the output at most
        rel = np.linalg.norm(o - outs[0][1], axis=-1) / np.linalg.norm(outs[0][1], axis=-1)
        assert rel.max() < 6e-3, rel.max()


def test_attention_split_count_invariance_many_rows():
    """The same with 256 query rows per KV head (8 row blocks) and a ragged last page."""
    outs = [attention_case("bf16", 64, 32, 8, 128, 64, 2048 + 40, 3, splits=s, stride=29) for s in (1, 2, 8, 16)]
    for worst, o, _ in outs:
        assert worst < ATT_REL["bf16"], worst
    for _, o, _ in outs[1:]:
        rel = np.linalg.norm(o - outs[0][1], axis=-1) / np.linalg.norm(outs[0][1], axis=-1)
        assert rel.max() < 6e-3, rel.max()


def test_kernels_are_run_to_run_identical():
    """Every MFMA kernel twice on the same inputs: bit-identical outputs.  (A vector instruction
    that reads matrix-core results before they have landed shows up here as last-bit noise long
    before it shows up in a tolerance.)"""
    import torch

    def twice(name, f):
        a = f(); torch.cuda.synchronize(); b = f(); torch.cuda.synchronize()
        assert torch.equal(a, b), name

    for M, N, K in [(1, 32000, 2048), (40, 3072, 2048), (32, 4096, 14336)]:
        a = binding.op_pack_tiled(to_dev(rnd(190, (M, K)), "bf16")[0])
        w = binding.op_pack_tiled(to_dev(rnd(191, (N, K), 0.05), "bf16")[0])
        w2 = binding.op_pack_tiled(to_dev(rnd(192, (N, K), 0.05), "bf16")[0])
        S = binding.op_linear_splits("bf16", M, N, K, True)
        twice(f"few-row linear {M} {N} {K}", lambda: binding.op_linear(a, w, S, tiled_shape=(M, N, K)))
        twice(f"few-row swiglu {M} {N} {K}", lambda: binding.op_linear_swiglu(a, w, w2, tiled_shape=(M, N, K)))
    for M, N, K in [(232, 2048, 2048), (3000, 4096, 512)]:
        a = binding.op_pack_tiled(to_dev(rnd(193, (M, K)), "bf16")[0])
        w = binding.op_pack_tiled(to_dev(rnd(194, (N, K), 0.05), "bf16")[0])
        twice(f"gemm {M} {N} {K}", lambda: binding.op_linear(a, w, 1, tiled_shape=(M, N, K)))
    pg = 64
    for Hq, Hkv, hd, P, rows, pos0 in [(32, 8, 64, 40, 40, 0), (32, 8, 128, 1024, 64, 960), (8, 2, 128, 330, 200, 130)]:
        npg = -(-P // pg)
        kp = to_dev(rnd(195, (npg, Hkv, pg * hd)), "bf16")[0]; vp = to_dev(rnd(196, (npg, Hkv, pg * hd)), "bf16")[0]
        q = to_dev(rnd(197, (rows, Hq, hd)), "bf16")[0]
        items = torch.tensor([[j, min(64, rows - j), pos0 + j, -1] for j in range(0, rows, 64)], dtype=torch.int32, device="cuda")
        twice(f"prefill attention {Hq} {Hkv} {hd} {P} {rows}",
              lambda: binding.op_attention_prefill(q, items, kp, vp, None, None, None, P, pg, False))
    for B, Hq, Hkv, hd, P, t in [(16, 32, 8, 64, 1000, 3), (32, 32, 8, 128, 4096, 200), (64, 40, 8, 128, 2048, 70)]:
        per = -(-t // pg)
        kp = to_dev(rnd(198, (-(-P // pg), Hkv, pg * hd)), "bf16")[0]; vp = to_dev(rnd(199, (-(-P // pg), Hkv, pg * hd)), "bf16")[0]
        ks = to_dev(rnd(200, (B * per, Hkv, pg * hd)), "bf16")[0]; vs = to_dev(rnd(201, (B * per, Hkv, pg * hd)), "bf16")[0]
        table = torch.arange(B * per, dtype=torch.int32, device="cuda").reshape(B, per)
        q = to_dev(rnd(202, (B, Hq, hd)), "bf16")[0]
        twice(f"decode attention {B} {Hq} {Hkv} {hd} {P} {t}",
              lambda: binding.op_attention_decode(q, kp, vp, ks, vs, table, P, t, pg))


def test_sample_op_cases():
    import torch
    V, B = 128256, 32
    lg = rnd(30, (B, V), 1.28)
    us = synth.uniforms(31, 1, (B,))
    ld, ud = torch.from_numpy(lg).cuda(), torch.from_numpy(us).cuda()
    toks, topk = binding.op_sample(ld, 0.7, 50, ud, want_topk=True)
    toks, topk = toks.cpu().numpy(), topk.cpu().numpy()
    ok = sum(check_sampler_on_logits(lg[b], 0.7, 50, us[b], toks[b], topk[b]) for b in range(B))
    assert ok >= B - 1
    # shared row: every candidate reads row 0
    t2 = binding.op_sample(ld, 0.7, 50, ud, shared_row=True).cpu().numpy()
    for b in range(B):
        check_sampler_on_logits(lg[0], 0.7, 50, us[b], t2[b])
    # all logits equal: the floor(u k)-th lowest id; k not a power of two; ties cut by id
    eq = torch.zeros((4, 4096), device="cuda")
    u4 = torch.tensor([0.0, 0.26, 0.5, 0.99], device="cuda")
    t3, k3 = binding.op_sample(eq, 0.7, 10, u4, want_topk=True)
    assert t3.cpu().tolist() == [0, 2, 5, 9] and k3.cpu().numpy().tolist() == [list(range(10))] * 4
    # duplicates straddling the cut, negative values, -0.0 vs +0.0
    row = np.array([1.0, -0.0, 0.0, 1.0, -3.0, 0.0, 1.0, 2.0] + [-9.0] * 56, np.float32)
    t4, k4 = binding.op_sample(torch.from_numpy(row[None]).cuda(), 1.0, 5, torch.tensor([0.999], device="cuda"), want_topk=True)
    assert k4.cpu().numpy().tolist() == [[7, 0, 3, 6, 1]]
    assert check_sampler_on_logits(row, 1.0, 5, 0.999, int(t4.cpu()[0]))
    # argmax, lowest id on ties
    g = binding.op_sample(torch.from_numpy(row[None]).cuda(), 0.0, 5, torch.tensor([0.5], device="cuda"))
    assert int(g.cpu()[0]) == 7
    g = binding.op_sample(eq, 1.0, 1, u4)
    assert g.cpu().tolist() == [0, 0, 0, 0]
    # u just below 1 -> last entry; tiny vocab below k
    small = torch.from_numpy(rnd(32, (2, 7))).cuda()
    t5, k5 = binding.op_sample(small, 0.9, 50, torch.tensor([1 - 2 ** -24, 0.0], device="cuda"), want_topk=True)
    assert k5.shape == (2, 7) and int(t5.cpu()[0]) == int(k5.cpu()[0, -1]) and int(t5.cpu()[1]) == int(k5.cpu()[1, 0])


@pytest.mark.parametrize("V,k,T,scale", [
    (128256, 1, 0.7, 1.28),        # k = 1 with T > 0: argmax path
    (128256, 2, 0.6, 1.28), (128256, 50, 0.6, 1.28), (128256, 64, 1.0, 0.01), (128256, 65, 0.7, 30.0),
    (128256, 400, 0.7, 1.28),      # 512 thread groups: the candidate list is near its capacity
    (128256, 1000, 0.7, 1.28),     # the list overflows: radix selection
    (128256, 4096, 1.3, 1.28),     # k above the fast path
    (4096, 50, 0.7, 1.0), (4100, 50, 0.7, 1.0), (4095, 50, 0.7, 1.0), (1000, 200, 0.7, 1.0),
])
def test_sample_selection_paths(V, k, T, scale):
    """Top-k ids bit-exact on both selection paths (threshold selection and radix selection),
    including rows quantised to few distinct values (many ties at the cut)."""
    import torch
    B = 3
    lg = rnd(33 + k, (B, V), scale)
    lg[1] = np.round(lg[1] * 4) / 4 if scale >= 1 else np.round(lg[1] * 400) / 400     # heavy ties
    lg[2, : V // 2] = lg[2, V // 2: 2 * (V // 2)]                                         # every value twice
    us = synth.uniforms(34, 1, (B,))
    print("case: sample paths", V, k, T, scale, flush=True)
    toks, topk = binding.op_sample(torch.from_numpy(lg).cuda(), T, k, torch.from_numpy(us).cuda(), want_topk=True)
    toks, topk = toks.cpu().numpy(), topk.cpu().numpy()
    for b in range(B):
        check_sampler_on_logits(lg[b], T, k, us[b], toks[b], topk[b])


def _top4_per_group(row):
    """Reference for the LM head's lists: ids of the four largest of every 64 consecutive logits
    under (value descending, id ascending)."""
    g = row.reshape(-1, 64).astype(np.float64)
    order = np.lexsort((np.broadcast_to(np.arange(64), g.shape), -g), axis=1)[:, :4]
    return order + 64 * np.arange(g.shape[0])[:, None]


@pytest.mark.parametrize("M,N,K", [(32, 65536, 256), (5, 131072, 512), (1, 65664, 256)])
def test_lm_head_top_lists(M, N, K):
    """The LM head's logits against the oracle's linear layer, and its per-group top lists against
    a plain selection on the device's own logits (ids and values bit-exact, ties by lower id:
    the weights are coarse so that equal logits are common)."""
    a = rnd(270, (M, K)); w = np.round(rnd(271, (N, K), 0.05) * 64) / 64
    ad, av = to_dev(a, "bf16"); wd, wv = to_dev(w, "bf16")
    if M == 5:                                     # rows of few distinct values: many ties inside a group
        av = np.sign(av); ad, av = to_dev(av, "bf16")
    print("case: lm head lists", M, N, K, flush=True)
    logits, lists = binding.op_lm_head(binding.op_pack_tiled(ad), binding.op_pack_tiled(wd), (M, N, K))
    logits, lists = logits.cpu().numpy(), lists.cpu().numpy()
    want = otf.linear(av, wv)
    np.testing.assert_allclose(logits, want, rtol=0, atol=2e-5 * np.abs(want).max() + 1e-6)
    for m in range(M):
        ids = _top4_per_group(logits[m])
        np.testing.assert_array_equal(lists[m, :, :, 1], ids)
        np.testing.assert_array_equal(lists[m, :, :, 0].view(np.float32) + 0.0, logits[m][ids] + 0.0)


def test_sample_with_top_lists():
    """Sampling from the LM head's lists instead of whole rows, on rows built to order (one-hot
    activations, so a row of logits is a row of bf16 weights, exactly): random rows at three
    scales (bf16 values tie often), a row whose largest values all sit in one group of 64 (the lists
    are inconclusive and the kernel must select from the whole row), a row of equal values, a row
    where exactly four of the top k share a group.  Ids and top-k lists equal the oracle sampler's
    on the device's logits for every temperature / k pair, with and without the lists in use."""
    import torch
    V, K, B = 65536, 256, 8
    rng = np.random.default_rng(272)
    rows = np.zeros((B, V), np.float32)
    rows[0] = rng.standard_normal(V) * 1.28
    rows[1] = rng.standard_normal(V) * 8.0
    rows[2] = rng.standard_normal(V) * 0.05
    rows[3] = rng.standard_normal(V); rows[3, 64 * 5: 64 * 5 + 40] += 9.0          # 40 of the top 50 in group 5
    rows[4] = 0.5                                                                    # all equal
    rows[5] = rng.standard_normal(V); rows[5, [700, 701, 702, 703]] = [9.0, 8.5, 8.0, 7.5]   # four of one group on top
    rows[6] = np.round(rng.standard_normal(V) * 2) / 2                               # few distinct values
    rows[7] = rng.standard_normal(V); rows[7, 64 * 900 + 3] = 30.0                   # one dominant id
    rows_d, rows_v = to_dev(rows, "bf16")
    a = np.zeros((B, K), np.float32); a[np.arange(B), np.arange(B)] = 1.0
    w = np.zeros((V, K), np.float32); w[:, :B] = rows_v.T
    ad, _ = to_dev(a, "bf16"); wd, _ = to_dev(w, "bf16")
    logits, lists = binding.op_lm_head(binding.op_pack_tiled(ad), binding.op_pack_tiled(wd), (B, V, K))
    lg = logits.cpu().numpy()
    np.testing.assert_array_equal(lg, rows_v)
    us = synth.uniforms(273, 1, (B,))
    ud = torch.from_numpy(us).cuda()
    for T, k in [(0.7, 50), (1.0, 64), (0.7, 65), (0.3, 2), (1.3, 5), (0.0, 50), (0.7, 1)]:
        print("case: sample lists", T, k, flush=True)
        toks, topk = binding.op_sample_lists(logits, lists, T, k, ud, want_topk=True)
        toks, topk = toks.cpu().numpy(), topk.cpu().numpy()
        for b in range(B):
            check_sampler_on_logits(lg[b], T, k, us[b], toks[b], topk[b])
        # the same ids as the whole-row sampler
        t2, k2 = binding.op_sample(logits, T, k, ud, want_topk=True)
        np.testing.assert_array_equal(topk, k2.cpu().numpy())
        np.testing.assert_array_equal(toks, t2.cpu().numpy())
    # every candidate reading row 0 of both
    t3 = binding.op_sample_lists(logits, lists, 0.7, 50, ud, shared_row=True).cpu().numpy()
    for b in range(B):
        check_sampler_on_logits(lg[0], 0.7, 50, us[b], t3[b])


def test_reward_score_op():
    import torch
    V, B, R = 128256, 64, 8
    lg = rnd(40, (B, V), 1.28)
    ids = synth.reward_token_ids(synth.WORKLOADS["8b-rerank"], R)
    vals = np.arange(R, dtype=np.float32)
    lp, sc, rk = binding.op_reward_score(torch.from_numpy(lg).cuda(), torch.from_numpy(ids).cuda(),
                                         torch.from_numpy(vals).cuda(), 0.7)
    lp, sc, rk = lp.cpu().numpy(), sc.cpu().numpy(), rk.cpu().numpy()
    want_lp = np.stack([osamp.reward_logprobs(lg[b], ids) for b in range(B)])
    np.testing.assert_allclose(lp, want_lp, rtol=0, atol=2e-5)
    want_sc = np.array([osamp.expected_value(want_lp[b], vals, 0.7) for b in range(B)])
    np.testing.assert_allclose(sc, want_sc, rtol=0, atol=2e-5)
    assert list(rk) == list(osamp.rank(sc))
    # equal reward logits with labels 0..4 -> exactly 2; ties ranked by index
    flat = np.zeros((3, 100), np.float32); flat[1, 50] = 5.0
    lp, sc, rk = binding.op_reward_score(torch.from_numpy(flat).cuda(), torch.arange(5, dtype=torch.int32, device="cuda"),
                                         torch.arange(5, dtype=torch.float32, device="cuda"), 1.0)
    assert sc.cpu().tolist() == [2.0, 2.0, 2.0] and rk.cpu().tolist() == [0, 1, 2]


# ---------------------------------------------------------------- tiled bf16 MFMA kernels
def test_pack_tiled_roundtrip():
    import torch
    for rows, K in [(32, 64), (33, 128), (100, 256), (4096, 512)]:
        t = torch.from_numpy(rnd(50, (rows, K))).to(torch.bfloat16).cuda()
        flat = binding.op_pack_tiled(t)
        assert flat.numel() == ((rows + 31) // 32 * 32) * K
        back = binding.tiled_to_rowmajor(flat.cpu(), rows, K)
        assert torch.equal(back, t.cpu())
        pad = binding.tiled_to_rowmajor(flat.cpu(), (rows + 31) // 32 * 32, K)[rows:]
        assert torch.all(pad == 0)


@pytest.mark.parametrize("M,N,K,S", [
    (32, 256, 512, 1), (32, 256, 512, 2), (16, 3072, 2048, 0), (1, 128, 256, 1), (33, 128, 1024, 2),
    (64, 384, 768, 1), (5, 6144, 4096, 0), (32, 4096, 14336, 0),
    (32, 128256, 4096, 0),         # the LM head of the 8B shape (two weight tiles per workgroup)
    (40, 65664, 256, 1),           # the same form with two row tiles of activations
    # 33..64 rows, enough weight tiles: four tiles per workgroup sharing the activations through LDS
    (64, 5120, 1024, 0), (33, 25600, 256, 1), (64, 3200, 2304, 0), (50, 20480, 512, 2), (64, 5120, 5120, 0),
    (65, 128, 256, 1), (200, 256, 512, 1), (130, 384, 1024, 1), (4096, 128, 256, 1),
    # 256-row-tile GEMM: ragged last row tile, a last band of fewer than 8 row tiles, padding ids
    (3000, 4096, 256, 1), (2300, 5632, 512, 1),
])
def test_linear_tiled(M, N, K, S):
    a = rnd(60, (M, K)); w = rnd(61, (N, K), 0.05)
    ad, av = to_dev(a, "bf16"); wd, wv = to_dev(w, "bf16")
    if S == 0:
        S = binding.op_linear_splits("bf16", M, N, K, True)
    print("case: linear tiled", M, N, K, S, flush=True)
    out = binding.op_linear(binding.op_pack_tiled(ad), binding.op_pack_tiled(wd), S, tiled_shape=(M, N, K))
    out = out.cpu().numpy().astype(np.float64).sum(0)
    want = otf.linear(av, wv)
    np.testing.assert_allclose(out, want, rtol=0, atol=2e-5 * np.abs(want).max() + 1e-6)


@pytest.mark.parametrize("M,N,K", [(3000, 4096, 256), (2300, 5632, 512), (70, 128, 256), (130, 384, 1024), (300, 640, 512)])
def test_linear_accumulate_tiled(M, N, K):
    """x += a w^T in the GEMM's epilogue (ragged last row tile, padding workgroup ids)."""
    import torch
    a = rnd(160, (M, K)); w = rnd(161, (N, K), 0.05); x = rnd(162, (M, N), 3.0)
    ad, av = to_dev(a, "bf16"); wd, wv = to_dev(w, "bf16")
    print("case: linear accumulate", M, N, K, flush=True)
    xd = torch.from_numpy(x.astype(np.float32)).cuda()
    binding.op_linear_accumulate(binding.op_pack_tiled(ad), binding.op_pack_tiled(wd), xd, (M, N, K))
    want = x.astype(np.float32).astype(np.float64) + otf.linear(av, wv)
    np.testing.assert_allclose(xd.cpu().numpy(), want, rtol=0, atol=2e-5 * np.abs(want).max() + 1e-6)


@pytest.mark.parametrize("rows,Hq,Hkv,hd,K", [
    (19, 4, 2, 64, 256),           # few rows: the weight-streaming kernel
    (64, 8, 2, 128, 512),
    (2100, 32, 8, 128, 256),       # many rows: the 256-row-tile GEMM (ragged last tile)
    (6200, 12, 2, 128, 256),       # N = 2048
    (100, 4, 2, 64, 256),          # one ragged row tile, N = 512
    (300, 5, 1, 128, 512),         # N = 896: an odd number of 128-column workgroups
    (19, 32, 8, 128, 256),         # few rows, N = 6144: the row-range form, 24 weight rows per workgroup
    (32, 12, 2, 128, 512),         # N = 2048: 8 rows per workgroup
    (5, 64, 8, 128, 256),          # N = 10240: 40 rows per workgroup (ranges that end on a tile edge and inside one)
])
def test_linear_qkv_rope_fused(rows, Hq, Hkv, hd, K):
    """QKV projection + rotation + query / key / value stores in one kernel, against the oracle's
    linear layer and rotation."""
    import torch
    pg, base, n_pos = 64, 500000.0, 5000
    nq = (Hq + 2 * Hkv) * hd
    a = rnd(170, (rows, K)); w = rnd(171, (nq, K), 0.05)
    ad, av = to_dev(a, "bf16"); wd, wv = to_dev(w, "bf16")
    rng = np.random.default_rng(172)
    pos = rng.integers(0, n_pos, rows).astype(np.int32)
    pos[:3] = [0, 1, n_pos - 1]
    n_pages = -(-rows // pg) + 1
    slots = rng.permutation(n_pages * pg)[:rows]
    page, off = (slots // pg).astype(np.int32), (slots % pg).astype(np.int32)
    kp = torch.zeros((n_pages, Hkv, pg * hd), dtype=torch.bfloat16, device="cuda")
    vp = torch.zeros((n_pages, Hkv, pg * hd), dtype=torch.bfloat16, device="cuda")
    print("case: fused qkv rope", rows, Hq, Hkv, hd, K, flush=True)
    q = binding.op_linear_qkv_rope(
        binding.op_pack_tiled(ad), binding.op_pack_tiled(binding.interleave_qk_rows(wd, Hq, Hkv, hd)), rows, K,
        torch.from_numpy(pos).cuda(), torch.from_numpy(page).cuda(), torch.from_numpy(off).cuda(),
        Hq, Hkv, hd, pg, base, n_pos, kp, vp)
    full = otf.linear(av, wv).reshape(rows, Hq + 2 * Hkv, hd)
    wq = otf.rope(full[:, :Hq], pos, base)
    wk = otf.rope(full[:, Hq:Hq + Hkv], pos, base)
    wvv = full[:, Hq + Hkv:]
    tol = TOL["bf16"] * np.abs(full).max()
    np.testing.assert_allclose(q.float().cpu().numpy(), wq, rtol=0, atol=tol)
    ku, vu = binding.kv_pages_unpack(kp, vp, pg, hd)
    kh, vh = ku.float().cpu().numpy(), vu.float().cpu().numpy()
    np.testing.assert_allclose(kh[page, :, off, :], wk, rtol=0, atol=tol)
    np.testing.assert_allclose(vh[page, :, off, :], wvv, rtol=0, atol=tol)
    written = np.zeros((n_pages, pg), bool); written[page, off] = True
    assert np.all(kh.transpose(0, 2, 1, 3)[~written] == 0) and np.all(vh.transpose(0, 2, 1, 3)[~written] == 0)


@pytest.mark.parametrize("M,N,K", [(32, 256, 512), (7, 14336, 4096), (64, 128, 256), (150, 256, 512),
                                   (3000, 2048, 512), (2070, 2944, 256), (65, 384, 256),
                                   (50, 27648, 512), (64, 20480, 256),
                                   # the row-range form: 56, 24, 8 and 48 weight rows per workgroup
                                   (32, 14336, 256), (17, 6144, 512), (1, 2048, 256), (30, 12288, 256)])
def test_linear_swiglu_tiled(M, N, K):
    a = rnd(62, (M, K)); wg = rnd(63, (N, K), 0.05); wu = rnd(64, (N, K), 0.05)
    ad, av = to_dev(a, "bf16"); gd, gv = to_dev(wg, "bf16"); ud, uv = to_dev(wu, "bf16")
    print("case: swiglu tiled", M, N, K, flush=True)
    flat = binding.op_linear_swiglu(binding.op_pack_tiled(ad), binding.op_pack_tiled(gd),
                                    binding.op_pack_tiled(ud), tiled_shape=(M, N, K))
    out = binding.tiled_to_rowmajor(flat.cpu(), M, N).float().numpy()
    want = otf.silu(otf.linear(av, gv)) * otf.linear(av, uv)
    np.testing.assert_allclose(out, want, rtol=0, atol=TOL["bf16"] * np.abs(want).max())


def test_scoring_size_gemms_on_sampled_rows():
    """The many-row GEMMs at the sizes one scoring chunk of the 8B shape launches (8192 rows):
    gate/up + SwiGLU 8192 x 14336 x 4096, down with the residual update 8192 x 4096 x 14336, QKV
    with rotation and page stores 8192 x 6144 x 4096.  The oracle computes 24 sampled rows of each
    (first, last, tile borders, random ones); every column of those rows is compared."""
    import torch
    M = 8192
    rng = np.random.default_rng(180)
    rows_s = np.unique(np.concatenate([[0, 31, 32, 255, 256, M - 257, M - 1], rng.integers(0, M, 17)]))
    # gate/up + SwiGLU
    d, F = 4096, 14336
    a = rnd(181, (M, d)); wg = rnd(182, (F, d), 0.02); wu = rnd(183, (F, d), 0.02)
    ad, av = to_dev(a, "bf16"); gd, gv = to_dev(wg, "bf16"); ud, uv = to_dev(wu, "bf16")
    print("case: scoring-size swiglu", flush=True)
    flat = binding.op_linear_swiglu(binding.op_pack_tiled(ad), binding.op_pack_tiled(gd), binding.op_pack_tiled(ud),
                                    tiled_shape=(M, F, d))
    act = binding.tiled_to_rowmajor(flat.cpu(), M, F)
    want = otf.silu(otf.linear(av[rows_s], gv)) * otf.linear(av[rows_s], uv)
    np.testing.assert_allclose(act[rows_s].float().numpy(), want, rtol=0, atol=TOL["bf16"] * np.abs(want).max())
    del gd, ud, flat
    # down projection adding to the residual stream; its input is the product above
    wd_ = rnd(184, (d, F), 0.02); x = rnd(185, (M, d), 2.0)
    dd, dv = to_dev(wd_, "bf16")
    print("case: scoring-size accumulate", flush=True)
    xd = torch.from_numpy(x.astype(np.float32)).cuda()
    actd = act.cuda()
    binding.op_linear_accumulate(binding.op_pack_tiled(actd), binding.op_pack_tiled(dd), xd, (M, d, F))
    want = x[rows_s].astype(np.float32).astype(np.float64) + otf.linear(act[rows_s].float().numpy(), dv)
    np.testing.assert_allclose(xd.cpu().numpy()[rows_s], want, rtol=0, atol=2e-5 * np.abs(want).max() + 1e-6)
    del dd, actd, xd
    # QKV + rotation + page stores
    Hq, Hkv, hd, pg, base, n_pos = 32, 8, 128, 64, 500000.0, 5120
    nq = (Hq + 2 * Hkv) * hd
    w = rnd(186, (nq, d), 0.02)
    wd2, wv = to_dev(w, "bf16")
    pos = rng.integers(0, n_pos, M).astype(np.int32)
    slots = rng.permutation((M // pg + 2) * pg)[:M]
    page, off = (slots // pg).astype(np.int32), (slots % pg).astype(np.int32)
    kp = torch.zeros((M // pg + 2, Hkv, pg * hd), dtype=torch.bfloat16, device="cuda")
    vp = torch.zeros_like(kp)
    print("case: scoring-size fused qkv rope", flush=True)
    q = binding.op_linear_qkv_rope(
        binding.op_pack_tiled(ad), binding.op_pack_tiled(binding.interleave_qk_rows(wd2, Hq, Hkv, hd)), M, d,
        torch.from_numpy(pos).cuda(), torch.from_numpy(page).cuda(), torch.from_numpy(off).cuda(),
        Hq, Hkv, hd, pg, base, n_pos, kp, vp)
    full = otf.linear(av[rows_s], wv).reshape(len(rows_s), Hq + 2 * Hkv, hd)
    tol = TOL["bf16"] * np.abs(full).max()
    np.testing.assert_allclose(q[torch.from_numpy(rows_s).cuda()].float().cpu().numpy(),
                               otf.rope(full[:, :Hq], pos[rows_s], base), rtol=0, atol=tol)
    ku, vu = binding.kv_pages_unpack(kp, vp, pg, hd)
    kh, vh = ku.float().cpu().numpy(), vu.float().cpu().numpy()
    np.testing.assert_allclose(kh[page[rows_s], :, off[rows_s], :], otf.rope(full[:, Hq:Hq + Hkv], pos[rows_s], base), rtol=0, atol=tol)
    np.testing.assert_allclose(vh[page[rows_s], :, off[rows_s], :], full[:, Hq + Hkv:], rtol=0, atol=tol)


def test_tiled_outputs_of_rmsnorm_and_attention():
    import torch
    for rows, d in [(37, 256), (1001, 512)]:      # the second: many rows, dealt to the XCDs in contiguous ranges
        x = rnd(65, (rows, d)); g = 1 + rnd(66, (d,), 0.1); p = rnd(67, (1, rows, d))
        gd, gv = to_dev(g, "bf16")
        h_plain = binding.op_add_rmsnorm(torch.from_numpy(x.copy()).cuda(), torch.from_numpy(p).cuda(), gd, 1e-6)
        xt = torch.from_numpy(x.copy()).cuda()
        h_tiled = binding.op_add_rmsnorm(xt, torch.from_numpy(p).cuda(), gd, 1e-6, tiled=True)
        assert torch.equal(binding.tiled_to_rowmajor(h_tiled.cpu(), rows, d), h_plain.cpu())
        want_x = x.astype(np.float64) + p[0]
        np.testing.assert_allclose(xt.cpu().numpy(), want_x, rtol=0, atol=1e-6)
        want_h = otf.rmsnorm(want_x, gv, 1e-6)
        np.testing.assert_allclose(h_plain.float().cpu().numpy(), want_h, rtol=0, atol=TOL["bf16"] * 4)
    # attention output, [B][Hq*hd] tiled
    B, Hq, Hkv, hd, pg, P, t = 5, 4, 2, 64, 16, 40, 9
    kpd, vpd, _, _ = make_pools("bf16", 3, Hkv, pg, hd, 70)
    ksd, vsd, _, _ = make_pools("bf16", B, Hkv, pg, hd, 72)
    table = torch.arange(B, dtype=torch.int32, device="cuda").reshape(B, 1)
    qd, _ = to_dev(rnd(74, (B, Hq, hd)), "bf16")
    o_plain = binding.op_attention_decode(qd, kpd, vpd, ksd, vsd, table, P, t, pg)
    o_tiled = binding.op_attention_decode(qd, kpd, vpd, ksd, vsd, table, P, t, pg, out_tiled=True)
    assert torch.equal(binding.tiled_to_rowmajor(o_tiled.cpu(), B, Hq * hd), o_plain.cpu().reshape(B, Hq * hd))


# ---------------------------------------------------------------- MFMA prefill / scoring attention
def prefill_case(Hq, Hkv, hd, P, seqs, stride=1, seed=90, out_tiled=False, item_rows=64, qscale=1.0, plant=()):
    """seqs: list of (pos_start, n_rows); pos_start < P means a prefix chunk (keys = prefix
    only, P grows to cover it), pos_start >= P a scored suffix starting at P.  plant: (row, head,
    key position) tuples: that key (a position the row can see) becomes 3 q[row, head].
    Returns (worst relative L2 error over the compared rows, errors of the planted rows)."""
    import torch
    pg = 64
    scoring = any(p0 >= P for p0, _ in seqs)
    n_pre = -(-P // pg)
    kpd, vpd, kpv, vpv = make_pools("bf16", n_pre, Hkv, pg, hd, seed)
    per = max(-(-max(n for _, n in seqs) // pg), 1)
    ksd, vsd, ksv, vsv = make_pools("bf16", len(seqs) * per, Hkv, pg, hd, seed + 2)
    table = np.random.default_rng(seed).permutation(len(seqs) * per).astype(np.int32).reshape(len(seqs), per)
    rows = sum(n for _, n in seqs)
    q = rnd(seed + 4, (rows, Hq, hd), qscale); qd, qv = to_dev(q, "bf16")
    G = Hq // Hkv
    seq_of_row = np.concatenate([np.full(n, si) for si, (_, n) in enumerate(seqs)]) if rows else np.zeros(0, int)
    for r, a, kpos in plant:
        if kpos < P:
            plant_key(kpv, vpv, kpd, vpd, kpos // pg, a // G, kpos % pg, qv[r, a], 3.0 / qscale, "bf16")
        else:
            j = kpos - P
            plant_key(ksv, vsv, ksd, vsd, table[seq_of_row[r], j // pg], a // G, j % pg, qv[r, a], 3.0 / qscale, "bf16")
    items, r0 = [], 0
    for si, (p0, n) in enumerate(seqs):
        for j in range(0, n, item_rows):
            items.append([r0 + j, min(item_rows, n - j), p0 + j, si if scoring else -1])
        r0 += n
    it = torch.tensor(items, dtype=torch.int32, device="cuda")
    print("case: prefill attention", Hq, Hkv, hd, P, seqs, plant, flush=True)
    out = binding.op_attention_prefill(qd, it, kpd, vpd, ksd if scoring else None, vsd if scoring else None,
                                       torch.from_numpy(table).cuda() if scoring else None, P, pg, out_tiled)
    if out_tiled:
        out = binding.tiled_to_rowmajor(out.cpu(), rows, Hq * hd).reshape(rows, Hq, hd)
    out = out.float().cpu().numpy()
    pos_of_row = np.concatenate([p0 + np.arange(n) for p0, n in seqs]) if rows else np.zeros(0, int)

    def want_row(r, a):
        si, pos, c = seq_of_row[r], pos_of_row[r], a // G
        keys = [kpv[:, c].reshape(-1, hd)[:min(P, pos + 1)]]
        vals = [vpv[:, c].reshape(-1, hd)[:min(P, pos + 1)]]
        if pos >= P:
            keys.append(ksv[table[si], c].reshape(-1, hd)[:pos - P + 1])
            vals.append(vsv[table[si], c].reshape(-1, hd)[:pos - P + 1])
        return otf.attention_one(qv[r, a], np.concatenate(keys), np.concatenate(vals))

    worst = 0.0
    for r in range(rows):
        for a in range(Hq):
            if (r * Hq + a) % stride == 0:
                worst = max(worst, rel_l2(out[r, a], want_row(r, a)))
    return worst, [rel_l2(out[r, a], want_row(r, a)) for r, a, _ in plant]


@pytest.mark.parametrize("Hq,Hkv,hd,P,seqs,stride,plant", [
    (8, 2, 128, 200, [(0, 200)], 1, [(199, 7, 150), (70, 0, 70)]),          # first prefill chunk, causal from position 0
    (8, 2, 64, 330, [(130, 200)], 1, [(199, 3, 5), (100, 6, 229)]),         # later chunk: earlier keys + own diagonal
    (32, 8, 128, 4096, [(2048, 2048)], 211, [(2047, 31, 4094), (1000, 5, 2000), (3, 12, 100)]),   # 8B shape, second half of the prefix
    (8, 2, 128, 150, [(150, 70), (150, 33), (150, 1)], 1, [(69, 1, 218), (90, 4, 149), (103, 7, 150)]),  # scoring: ragged suffixes
    (40, 8, 128, 1000, [(1000, 100), (1000, 64)], 7, [(99, 39, 999), (163, 20, 1063)]),            # 5 query heads per KV head
    (32, 8, 128, 4096, [(4096, 1024)] * 3, 1531, [(1023, 0, 5119), (2047, 31, 4000), (3071, 9, 5000), (2500, 17, 4500)]),  # reranking shape
    (4, 4, 64, 1, [(1, 65)], 1, [(64, 2, 65)]),
])
def test_attention_prefill_mfma(Hq, Hkv, hd, P, seqs, stride, plant):
    """Every compared row within the relative bound, and rows one of whose keys (late in the
    prefix, in the row's own suffix page, on its own diagonal) decides the output."""
    worst, planted = prefill_case(Hq, Hkv, hd, P, seqs, stride, plant=plant)
    assert worst < ATT_REL["bf16"], worst
    assert max(planted) < ATT_REL["bf16"], planted


@pytest.mark.parametrize("item_rows", [32, 48, 17])
def test_attention_prefill_item_sizes(item_rows):
    """Items shorter than 64 positions: the second half of the workgroup has fewer rows or none."""
    worst, _ = prefill_case(8, 2, 128, 150, [(150, 130), (150, 33)], item_rows=item_rows)
    assert worst < ATT_REL["bf16"], worst
    worst, _ = prefill_case(8, 2, 64, 200, [(0, 200)], item_rows=item_rows)
    assert worst < ATT_REL["bf16"], worst


def test_attention_prefill_tiled_output_matches():
    a, _ = prefill_case(8, 2, 128, 100, [(100, 40), (100, 9)], out_tiled=True)
    assert a < ATT_REL["bf16"], a


@pytest.mark.parametrize("qscale", [8.0, 0.01])
def test_attention_with_peaked_and_flat_softmax(qscale):
    """Scores with a standard deviation of ~90 (one key takes nearly all the weight, the running
    maximum jumps far past the lazy rescale threshold several times) and of ~0.1 (uniform
    weights), on both MFMA attention kernels."""
    worst, _, _ = attention_case("bf16", 9, 8, 2, 128, 64, 700, 130, qscale=qscale, stride=3)
    assert worst < 2 * ATT_REL["bf16"], worst
    worst, _, _ = attention_case("bf16", 4, 4, 4, 64, 64, 0, 257, qscale=qscale)
    assert worst < 2 * ATT_REL["bf16"], worst
    worst, _ = prefill_case(8, 2, 128, 150, [(150, 130)], qscale=qscale, stride=3)
    assert worst < 2 * ATT_REL["bf16"], worst


def test_mfma_probe_counts_what_it_claims():
    """All-ones operands: every accumulator element gains 16 per MFMA, so a thread's 8 tiles x 16
    registers sum to 8 * 16 * 16 * iters."""
    import torch
    n_wg, iters = 3, 5
    ops = torch.ones(n_wg * 256 * 48, dtype=torch.bfloat16, device="cuda")
    out = torch.empty(n_wg * 256, dtype=torch.float32, device="cuda")
    lib = binding.load_library()
    assert lib.mc_op_mfma_probe(None, ops.data_ptr(), out.data_ptr(), n_wg, iters) == 0
    torch.cuda.synchronize()
    assert torch.all(out == 8 * 16 * 16 * iters)
    assert binding.op_mfma_probe(ops, n_wg, iters) == n_wg * 4 * iters * 8 * 32768.0
