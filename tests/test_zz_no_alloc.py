"""The decode-attention entry point that allocates nothing (the library's own static scratch
buffer) against the entry point that takes a caller's workspace: same kernels, so the outputs
must be bit-identical; two calls in a row, the second on a smaller input, so that what the first
call left in the shared buffer must not leak into the second."""
import numpy as np
import pytest

from oracle import transformer as otf
from paper_2601_05475_amd import binding, synth

pytestmark = pytest.mark.gpu


def _case(dtype, B, Hq, Hkv, hd, pg, P, t, seed):
    import torch
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    n_pre, per = -(-P // pg), -(-t // pg)

    def pool(n, sd):
        k = torch.from_numpy(synth.normal(sd, 9, (n, Hkv, pg, hd), 0.0, 1.0, "f32")).to(tdt).cuda()
        v = torch.from_numpy(synth.normal(sd + 1, 9, (n, Hkv, pg, hd), 0.0, 1.0, "f32")).to(tdt).cuda()
        return binding.kv_pages_pack(k, v) + (k.float().cpu().numpy(), v.float().cpu().numpy())

    kp, vp, kpv, vpv = pool(n_pre, seed)
    ks, vs, ksv, vsv = pool(B * per, seed + 2)
    table = np.random.default_rng(seed).permutation(B * per).astype(np.int32).reshape(B, per)
    q = torch.from_numpy(synth.normal(seed + 4, 9, (B, Hq, hd), 0.0, 1.0, "f32")).to(tdt).cuda()
    return dict(q=q, kp=kp, vp=vp, ks=ks, vs=vs, table=torch.from_numpy(table).cuda(), P=P, t=t, pg=pg,
                host=(q.float().cpu().numpy(), kpv, vpv, ksv, vsv, table))


def _run(c, static):
    import torch
    out = torch.empty_like(c["q"])
    binding.op_attention_decode(c["q"], c["kp"], c["vp"], c["ks"], c["vs"], c["table"], c["P"], c["t"], c["pg"],
                                out=out, static_scratch=static)
    return out


def _oracle_rows(c, rows):
    qv, kpv, vpv, ksv, vsv, table = c["host"]
    Hq, hd = qv.shape[1], qv.shape[2]
    G = Hq // kpv.shape[1]
    per = -(-c["t"] // c["pg"])
    out = []
    for b, a in rows:
        kvh = a // G
        keys = np.concatenate([kpv[:, kvh].reshape(-1, hd)[:c["P"]], ksv[table[b, :per], kvh].reshape(-1, hd)[:c["t"]]])
        vals = np.concatenate([vpv[:, kvh].reshape(-1, hd)[:c["P"]], vsv[table[b, :per], kvh].reshape(-1, hd)[:c["t"]]])
        out.append(otf.attention_one(qv[b, a], keys, vals))
    return np.stack(out)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_scratch_entry_point_equals_the_workspace_one(dtype):
    import torch
    big = _case(dtype, 32, 32, 8, 128, 64, 4096 if dtype == "bf16" else 256, 130, 300)
    small = _case(dtype, 3, 8, 2, 128, 64, 200, 70, 310)
    print("case: static scratch", dtype, flush=True)
    got = []
    for c in (big, small):                       # back to back on one stream, the smaller input second
        got.append(_run(c, static=True))
    torch.cuda.synchronize()
    for c, g in zip((big, small), got):
        want = _run(c, static=False)
        torch.cuda.synchronize()
        assert torch.equal(g, want)
        rows = [(0, 0), (c["q"].shape[0] - 1, c["q"].shape[1] - 1), (c["q"].shape[0] // 2, 3)]
        ref = _oracle_rows(c, rows)
        have = np.stack([g[b, a].float().cpu().numpy() for b, a in rows])
        rel = np.linalg.norm(have - ref, axis=1) / np.linalg.norm(ref, axis=1)
        assert rel.max() < (1e-5 if dtype == "f32" else 1e-2), rel


def test_static_scratch_rejects_what_does_not_fit():
    import torch
    lib = binding.load_library()
    need = lib.mc_op_attention_decode_ws(64, 40, 8, 128, 16384, 1024, 64)
    assert need > 32 << 20
    q = torch.zeros((64, 40, 128), dtype=torch.bfloat16, device="cuda")
    kp = torch.zeros((256, 8, 64 * 128), dtype=torch.bfloat16, device="cuda")
    ks = torch.zeros((64 * 16, 8, 64 * 128), dtype=torch.bfloat16, device="cuda")
    table = torch.arange(64 * 16, dtype=torch.int32, device="cuda").reshape(64, 16)
    with pytest.raises(binding.McError) as e:
        binding.op_attention_decode(q, kp, kp, ks, ks, table, 16384, 1024, 64, static_scratch=True)
    assert e.value.code == -5
