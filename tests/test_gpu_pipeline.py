"""R-worker for N blocks and two mini-batches on two streams (FastDecode Section 4.1): every
block of every token step is checked against the oracle, which keeps its own host copy of each
(mini-batch, block) cache.  Bar as elsewhere: lengths and cache bytes bit-exact, out within
2e-3 * max|V|."""
import numpy as np
import pytest
import torch

from oracle import rpart_oracle as O
from paper_2403_11421_amd import rpart, workloads as W
from paper_2403_11421_amd.pipeline import RWorker
from tests.util import bits, f64

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _vectors(cfg, which, mb, layer, token, dev):
    """fp16 [B, H, d]; a distinct seed per (mini-batch, block, token step)."""
    return W.gen_vectors(cfg, which, seed=1000 + 97 * mb + 13 * layer + token, device=dev)


def _tm(t):
    """device [H, cap, ...] -> host token-major [cap, H, ...]"""
    return np.ascontiguousarray(t.permute(1, 0, *range(2, t.dim())).cpu().numpy())


def _tm16(t):
    """fp16 device block -> host token-major bit patterns"""
    return bits(t.permute(1, 0, 2))


@pytest.mark.parametrize("n_streams", [2, 1])
@pytest.mark.parametrize("kv", ["fp16", "int8", "int4"])
def test_every_block_of_every_token_matches_the_oracle(kv, n_streams):
    dev = "cuda"
    H, d, N, n_tokens = 3, 128, 3, 3
    lens0 = [[0, 5, 300, 64, 1500, 33], [700, 1, 129, 0]]           # two ragged mini-batches
    cfgs = [W.RPartConfig(f"mb{m}", len(l), H, d, "const", 0, 0) for m, l in enumerate(lens0)]
    caps = [[L + n_tokens for L in l] for l in lens0]
    rw = RWorker(H, d, N, caps, kv=kv, n_streams=n_streams)
    host = {}
    for m, cfg in enumerate(cfgs):
        for layer in range(N):
            c = rw.caches[m][layer]
            for b, L in enumerate(lens0[m]):
                if L:
                    c.fill("K", b, W.gen_cache_block(cfg, "K", b, L, seed=7 + layer, device=dev))
                    c.fill("V", b, W.gen_cache_block(cfg, "V", b, L, seed=8 + layer, device=dev))
            c.set_lens(lens0[m])
            if kv == "fp16":
                host[m, layer] = dict(K=[_tm16(c.block("K", b)) for b in range(cfg.B)],
                                      V=[_tm16(c.block("V", b)) for b in range(cfg.B)],
                                      lens=np.asarray(lens0[m], np.int32))
            else:
                host[m, layer] = dict(Kc=[_tm(c.codes("K", b)) for b in range(cfg.B)],
                                      Ks=[_tm(c.scales("K", b)) for b in range(cfg.B)],
                                      Vc=[_tm(c.codes("V", b)) for b in range(cfg.B)],
                                      Vs=[_tm(c.scales("V", b)) for b in range(cfg.B)],
                                      lens=np.asarray(lens0[m], np.int32))

    for token in range(n_tokens):
        q = [[_vectors(cfgs[m], "q", m, l, token, dev) for l in range(N)] for m in range(2)]
        kn = [[_vectors(cfgs[m], "k_new", m, l, token, dev) for l in range(N)] for m in range(2)]
        vn = [[_vectors(cfgs[m], "v_new", m, l, token, dev) for l in range(N)] for m in range(2)]
        out = [[torch.full((cfgs[m].B, H, d), float("nan"), dtype=torch.float16, device=dev)
                for _ in range(N)] for m in range(2)]
        torch.cuda.synchronize()
        rw.token_step(q, kn, vn, out)
        torch.cuda.synchronize()
        assert rw.status() == 0
        for m in range(2):
            for layer in range(N):
                h = host[m, layer]
                c = rw.caches[m][layer]
                qb, kb, vb = (bits(t[m][layer].cpu()) for t in (q, kn, vn))
                if kv == "fp16":
                    O.kv_append(h["K"], h["V"], h["lens"], kb, vb)
                    want, _, _ = O.rpart_decode(h["K"], h["V"], h["lens"], qb)
                    maxv = max(float(np.abs(f64(v[:L])).max()) for v, L in zip(h["V"], h["lens"]) if L)
                    for b in range(cfgs[m].B):
                        assert np.array_equal(_tm16(c.block("K", b)), h["K"][b])
                        assert np.array_equal(_tm16(c.block("V", b)), h["V"][b])
                else:
                    if kv == "int8":
                        O.kvq_append(h["Kc"], h["Ks"], h["Vc"], h["Vs"], h["lens"], kb, vb)
                        want, _ = O.rpartq_decode(h["Kc"], h["Ks"], h["Vc"], h["Vs"], h["lens"], qb)
                        maxv = max(float(np.abs((vc[:L].astype(np.float64) - 128) * vs[:L, :, None]).max())
                                   for vc, vs, L in zip(h["Vc"], h["Vs"], h["lens"]) if L)
                    else:                                    # 4 bit: packed codes, (scale, zero) pairs
                        O.kvq4_append(h["Kc"], h["Ks"], h["Vc"], h["Vs"], h["lens"], kb, vb)
                        want, _ = O.rpartq4_decode(h["Kc"], h["Ks"], h["Vc"], h["Vs"], h["lens"], qb)
                        maxv = max(float(np.abs(O.unpack_u4(vc[:L]).astype(np.float64) * vs[:L, :, 0:1]
                                                + vs[:L, :, 1:2]).max())
                                   for vc, vs, L in zip(h["Vc"], h["Vs"], h["lens"]) if L)
                    for b in range(cfgs[m].B):
                        assert np.array_equal(_tm(c.codes("K", b)), h["Kc"][b])
                        assert np.array_equal(_tm(c.scales("K", b)), h["Ks"][b])
                        assert np.array_equal(_tm(c.codes("V", b)), h["Vc"][b])
                        assert np.array_equal(_tm(c.scales("V", b)), h["Vs"][b])
                assert np.array_equal(c.seq_lens.cpu().numpy(), h["lens"])
                got = out[m][layer].cpu().double().numpy()
                assert np.all(np.isfinite(got))
                err = float(np.abs(got - want).max())
                assert err <= TOL * maxv, (kv, token, m, layer, err, maxv)
        # every block planned from block 0's lengths: the plan's token total is this step's
        for m in range(2):
            assert rpart.fd_plan_info(rw.ws[m])["total_tokens"] == int(host[m, 0]["lens"].sum())


def test_layer_step_rejects_bad_arguments():
    rw = RWorker(2, 128, 1, [[4, 4]], n_streams=1)
    c = rw.caches[0][0]
    x = torch.zeros(2, 2, 128, dtype=torch.float16, device="cuda")
    with pytest.raises(rpart.FdError) as e:
        rpart.fd_rpart_layer_step(c.desc, x, x, x, x, rw.ws[0][:64], True)
    assert e.value.code == rpart.FD_EWORKSPACE
    with pytest.raises(rpart.FdError) as e:
        rpart.fd_rpart_layer_step(c.desc, x, None, x, x, rw.ws[0], True)
    assert e.value.code == rpart.FD_EINVAL
    torch.cuda.synchronize()
    assert c.seq_lens.cpu().tolist() == [0, 0]              # a failing call enqueues nothing
