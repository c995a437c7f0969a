"""GPU parity of rvq_attn_decode (attention of one query position over a cache of codes) against
the fp64 oracle, through the C ABI.

Tolerance.  Keys, values and scores are fp32 on the GPU.  A score s = scale * q . k carries an
absolute error of about 2^-23 * (number of terms) * sum |q_c k_c| <= 3e-5 for the |s| <= 60 seen
here, which turns into a relative error of the same size in the softmax weight exp(s - max); the
value sum adds 2^-23 per term.  The bar: per query head max |gpu - oracle| <= 1e-4 * max |oracle|
(measured errors are printed; they are 1e-7 to 2e-6)."""
import numpy as np
import pytest

import oracle
from test_gpu_parity import _b, _torch

pytestmark = pytest.mark.gpu

HD, G = 128, 4


def _case(seed, N, Hkv, rep, depth, Kk, Kv, kgroup, vgroup, std_dtype="fp16", scale_flag=1, rope=True,
          sharp=1.0):
    rng = np.random.Generator(np.random.PCG64(seed))
    Ck = (rng.standard_normal((depth, Kk, 32)) * (0.6 ** np.arange(depth))[:, None, None]).astype(np.float32)
    Cv = (rng.standard_normal((depth, Kv, 32)) * (0.6 ** np.arange(depth))[:, None, None]).astype(np.float32)
    rows = N * Hkv
    kc = rng.integers(0, Kk, (rows, G, depth)).astype(np.int16)
    vc = rng.integers(0, Kv, (rows, G, depth)).astype(np.int16)
    sdt = np.float16 if std_dtype == "fp16" else np.float32
    ks = np.exp(0.5 * rng.standard_normal(rows)).astype(sdt) if scale_flag else None
    vs = np.exp(0.5 * rng.standard_normal(rows)).astype(sdt) if scale_flag else None
    q = (sharp * rng.standard_normal((Hkv * rep, HD))).astype(np.float32)
    if rope:
        cos, sin = oracle.rope_tables(np.arange(N) + int(rng.integers(0, 1000)), HD)
        cos, sin = cos.astype(np.float32), sin.astype(np.float32)
    else:
        cos = sin = None
    return dict(N=N, Hkv=Hkv, rep=rep, depth=depth, Kk=Kk, Kv=Kv, kgroup=kgroup, vgroup=vgroup,
                Ck=Ck, Cv=Cv, kc=kc, vc=vc, ks=ks, vs=vs, q=q, cos=cos, sin=sin, std_dtype=std_dtype,
                scale_flag=scale_flag)


def _run_gpu(c, scale):
    torch, b = _torch(), _b()
    sd = b.F16 if c["std_dtype"] == "fp16" else b.F32
    kq = b.Quantizer(d=HD, dhat=32, depth=c["depth"], K=c["Kk"], grouping=c["kgroup"], std_dtype=sd,
                     scale=c["scale_flag"])
    vq = b.Quantizer(d=HD, dhat=32, depth=c["depth"], K=c["Kv"], grouping=c["vgroup"], std_dtype=sd,
                     scale=c["scale_flag"])
    kq.set_codebooks(torch.from_numpy(c["Ck"]).cuda())
    vq.set_codebooks(torch.from_numpy(c["Cv"]).cuda())
    dev = lambda a: None if a is None else torch.from_numpy(a).cuda()
    Hq = c["Hkv"] * c["rep"]
    wsb = b.rvq_attn_workspace_bytes(c["N"], Hq, c["Hkv"])
    ws = torch.empty(wsb // 4, dtype=torch.float32, device="cuda")
    out = torch.full((Hq, HD), float("nan"), dtype=torch.float32, device="cuda")
    args = [dev(c["q"]), Hq, c["Hkv"], dev(c["kc"]), dev(c["ks"]), dev(c["vc"]), dev(c["vs"]), c["N"],
            dev(c["cos"]), dev(c["sin"]), scale, out, ws, wsb]
    b.rvq_attn_decode(kq.ctx, vq.ctx, *args)
    torch.cuda.synchronize()
    res = out.cpu().numpy().astype(np.float64)
    kq.close()
    vq.close()
    return res


def _run_oracle(c, scale):
    N = c["N"]
    one = np.ones((N, HD // 2)) if c["cos"] is None else c["cos"]
    zero = np.zeros((N, HD // 2)) if c["sin"] is None else c["sin"]
    rows = N * c["Hkv"]
    ks = np.ones(rows) if c["ks"] is None else c["ks"]
    vs = np.ones(rows) if c["vs"] is None else c["vs"]
    return oracle.attn_decode(c["q"], c["kc"], ks, c["Ck"], c["kgroup"], c["vc"], vs, c["Cv"], c["vgroup"],
                              one, zero, scale, c["Hkv"])


def _check(c, scale=1.0 / np.sqrt(HD), tol=1e-4):  # measured: <= 2e-6
    got = _run_gpu(c, scale)
    want = _run_oracle(c, scale)
    assert np.isfinite(got).all()
    err = np.abs(got - want).max(axis=1) / np.abs(want).max(axis=1)
    assert err.max() <= tol, "relative error per query head: %s" % err
    return float(err.max())


@pytest.mark.parametrize("case", [
    # N, Hkv, rep, depth, Kk, Kv, key grouping, value grouping, std type, scaled, rotation
    (300, 2, 4, 8, 256, 300, oracle.STRIDED, oracle.CONTIGUOUS, "fp16", 1, True),   # the paper's setting, ragged N
    (1, 3, 1, 8, 64, 64, oracle.STRIDED, oracle.CONTIGUOUS, "fp16", 1, True),       # one token: its value
    (7, 1, 2, 8, 64, 64, oracle.CONTIGUOUS, oracle.STRIDED, "fp32", 1, True),       # fewer tokens than a trip
    (1029, 2, 8, 6, 100, 33, oracle.CONTIGUOUS, oracle.CONTIGUOUS, "fp16", 1, True),  # depth 6: record of 12 bytes
    (2500, 4, 2, 4, 1024, 2048, oracle.STRIDED, oracle.STRIDED, "fp16", 1, False),  # no rotation
    (777, 2, 4, 1, 17, 5, oracle.STRIDED, oracle.CONTIGUOUS, "fp16", 0, True),      # one stage, rows not scaled
    (40000, 8, 4, 8, 2048, 2048, oracle.STRIDED, oracle.CONTIGUOUS, "fp16", 1, True),  # several splits per head
    # the compile-time fast case (depth 8, tables, fp16 std) in its other instantiations
    (513, 2, 8, 8, 128, 128, oracle.CONTIGUOUS, oracle.STRIDED, "fp16", 1, True),
    (2000, 3, 2, 8, 500, 700, oracle.CONTIGUOUS, oracle.CONTIGUOUS, "fp16", 1, True),
    (900, 2, 1, 8, 2048, 2048, oracle.STRIDED, oracle.STRIDED, "fp16", 1, True),
])
def test_attn_decode_against_oracle(gpu_device, case):
    N, Hkv, rep, depth, Kk, Kv, kg, vg, sdt, sc, rope = case
    c = _case(1000 + N, N, Hkv, rep, depth, Kk, Kv, kg, vg, sdt, sc, rope)
    e = _check(c)
    print("N=%d Hkv=%d rep=%d depth=%d: max relative error %.2e" % (N, Hkv, rep, depth, e))


def test_attn_decode_sharp_and_flat_softmax(gpu_device):
    """Queries scaled up until one token takes nearly all the weight, and scale 0 (the mean of the
    values): the running maximum and the merges of half-wavefronts and splits must hold in both."""
    c = _case(77, 5000, 2, 4, 8, 512, 512, oracle.STRIDED, oracle.CONTIGUOUS, sharp=12.0)
    _check(c)
    c2 = _case(78, 5000, 2, 4, 8, 512, 512, oracle.STRIDED, oracle.CONTIGUOUS)
    got = _run_gpu(c2, 0.0)
    vx = oracle.decode(c2["vc"], c2["vs"], c2["Cv"], HD, oracle.CONTIGUOUS).reshape(5000, 2, HD).mean(0)
    for a in range(8):
        np.testing.assert_allclose(got[a], vx[a // 4], rtol=1e-4, atol=1e-5 * np.abs(vx).max())


def test_attn_decode_equals_decode_then_attention_on_the_gpu(gpu_device):
    """The fused call against the unfused route through the library's own decode entry points
    (rvq_decode_rope for keys, rvq_decode for values, fp32 outputs) followed by a plain softmax
    attention in torch: the same numbers to fp32 accuracy."""
    torch, b = _torch(), _b()
    c = _case(5, 4096, 4, 4, 8, 2048, 2048, oracle.STRIDED, oracle.CONTIGUOUS)
    scale = 1.0 / np.sqrt(HD)
    got = _run_gpu(c, scale)
    kq = b.Quantizer(d=HD, dhat=32, depth=8, K=2048, grouping=b.STRIDED, std_dtype=b.F16, out_dtype=b.F32)
    vq = b.Quantizer(d=HD, dhat=32, depth=8, K=2048, grouping=b.CONTIGUOUS, std_dtype=b.F16, out_dtype=b.F32)
    kq.set_codebooks(torch.from_numpy(c["Ck"]).cuda())
    vq.set_codebooks(torch.from_numpy(c["Cv"]).cuda())
    rows = c["N"] * c["Hkv"]
    cosr = torch.from_numpy(np.repeat(c["cos"], c["Hkv"], axis=0)).cuda()
    sinr = torch.from_numpy(np.repeat(c["sin"], c["Hkv"], axis=0)).cuda()
    kx = torch.empty((rows, HD), dtype=torch.float32, device="cuda")
    vx = torch.empty((rows, HD), dtype=torch.float32, device="cuda")
    b.rvq_decode_rope(kq.ctx, torch.from_numpy(c["kc"]).cuda(), torch.from_numpy(c["ks"]).cuda(), rows, 8,
                      cosr, sinr, HD, kx, HD)
    b.rvq_decode(vq.ctx, torch.from_numpy(c["vc"]).cuda(), torch.from_numpy(c["vs"]).cuda(), rows, 8, vx, HD)
    kx = kx.view(c["N"], c["Hkv"], HD).double()
    vx = vx.view(c["N"], c["Hkv"], HD).double()
    qd = torch.from_numpy(c["q"]).cuda().double()
    for a in range(c["Hkv"] * c["rep"]):
        h = a // c["rep"]
        p = torch.softmax(scale * (kx[:, h] @ qd[a]), dim=0)
        want = (p @ vx[:, h]).cpu().numpy()
        np.testing.assert_allclose(got[a], want, rtol=0, atol=1e-4 * np.abs(want).max())
    kq.close()
    vq.close()


def test_attn_decode_error_codes(gpu_device):
    torch, b = _torch(), _b()
    c = _case(9, 64, 2, 4, 8, 64, 64, oracle.STRIDED, oracle.CONTIGUOUS)
    kq = b.Quantizer(d=HD, dhat=32, depth=8, K=64, grouping=b.STRIDED)
    vq = b.Quantizer(d=HD, dhat=32, depth=8, K=64, grouping=b.CONTIGUOUS)
    wide = b.Quantizer(d=256, dhat=32, depth=8, K=64)
    dev = lambda a: torch.from_numpy(a).cuda()
    q, kc, ks, vc, vs = dev(c["q"]), dev(c["kc"]), dev(c["ks"]), dev(c["vc"]), dev(c["vs"])
    cos, sin = dev(c["cos"]), dev(c["sin"])
    out = torch.empty((8, HD), device="cuda")
    wsb = b.rvq_attn_workspace_bytes(64, 8, 2)
    ws = torch.empty(wsb // 4, device="cuda")
    st = torch.cuda.current_stream().cuda_stream

    def call(kctx=None, vctx=None, Hq=8, Hkv=2, N=64, wsbytes=wsb, cosp=cos, sinp=sin, packed=0):
        p = lambda t: None if t is None else t.data_ptr()
        return b.lib.rvq_attn_decode(kctx or kq.ctx, vctx or vq.ctx, p(q), Hq, Hkv, p(kc), p(ks), p(vc), p(vs),
                                     packed, N, p(cosp), p(sinp), 0.1, p(out), p(ws), wsbytes, st)

    assert call() == b.RVQ_ENOCODEBOOK
    kq.set_codebooks(dev(c["Ck"]))
    vq.set_codebooks(dev(c["Cv"]))
    assert call() == b.RVQ_OK
    assert call(N=0) == b.RVQ_EINVAL                   # a softmax over nothing
    assert call(Hq=6) == b.RVQ_EINVAL                  # three query heads per kv head
    assert call(Hq=7) == b.RVQ_EINVAL
    assert call(kctx=wide.ctx) == b.RVQ_EINVAL         # heads must have 128 channels
    assert call(wsbytes=wsb - 4) == b.RVQ_EWORKSPACE
    assert call(sinp=None) == b.RVQ_EINVAL             # one table without the other
    assert call(packed=1) == b.RVQ_EINVAL              # 6-bit codes (K = 64) are not read in place
    assert call(packed=2) == b.RVQ_EINVAL
    assert b.rvq_attn_workspace_bytes(0, 8, 2) == 0
    torch.cuda.synchronize()
    for x in (kq, vq, wide):
        x.close()


@pytest.mark.parametrize("case", [
    # N, Hkv, rep, K, key grouping, value grouping, rotation, std type
    (3001, 2, 4, 2048, oracle.STRIDED, oracle.CONTIGUOUS, True, "fp16"),   # 11-bit codes, the fast case
    (1000, 3, 2, 4096, oracle.CONTIGUOUS, oracle.STRIDED, True, "fp16"),   # 12-bit codes
    (700, 1, 8, 1500, oracle.STRIDED, oracle.STRIDED, False, "fp32"),      # 11 bits, run-time conditions
])
def test_attn_decode_from_packed_records(gpu_device, case):
    """The cache as rvq_pack_codes stores it (11 or 12 bits per code): the same output, bit for bit,
    as from the int16 codes, and the oracle's bar against the fp64 definition."""
    torch, b = _torch(), _b()
    N, Hkv, rep, K, kg, vg, rope, sdt = case
    c = _case(4000 + N, N, Hkv, rep, 8, K, K, kg, vg, sdt, 1, rope)
    scale = 1.0 / np.sqrt(HD)
    want = _run_oracle(c, scale)
    sd = b.F16 if sdt == "fp16" else b.F32
    kq = b.Quantizer(d=HD, dhat=32, depth=8, K=K, grouping=kg, std_dtype=sd)
    vq = b.Quantizer(d=HD, dhat=32, depth=8, K=K, grouping=vg, std_dtype=sd)
    kq.set_codebooks(torch.from_numpy(c["Ck"]).cuda())
    vq.set_codebooks(torch.from_numpy(c["Cv"]).cuda())
    dev = lambda a: None if a is None else torch.from_numpy(a).cuda()
    kc, vc = dev(c["kc"]), dev(c["vc"])
    kp, vp = kq.pack(kc), vq.pack(vc)
    assert kp.shape[-1] == (11 if K <= 2048 else 12)
    Hq = Hkv * rep
    wsb = b.rvq_attn_workspace_bytes(N, Hq, Hkv)
    ws = torch.empty(wsb // 4, dtype=torch.float32, device="cuda")
    outs = []
    for codes_k, codes_v, packed in ((kc, vc, 0), (kp, vp, 1)):
        out = torch.full((Hq, HD), float("nan"), dtype=torch.float32, device="cuda")
        b.rvq_attn_decode(kq.ctx, vq.ctx, dev(c["q"]), Hq, Hkv, codes_k, dev(c["ks"]), codes_v, dev(c["vs"]), N,
                          dev(c["cos"]), dev(c["sin"]), scale, out, ws, wsb, packed=packed)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])
    err = np.abs(outs[1] - want).max(axis=1) / np.abs(want).max(axis=1)
    assert err.max() <= 1e-4, err
    kq.close()
    vq.close()
