"""GPU parity at the full sizes of the workloads, and the instantiations that only those sizes
reach: codebooks larger than the 2048 codewords LDS holds swept by workgroups that walk several
chunks, workload 5 (N = 131072 x 4096 channels, K = 4096) end to end, workload 4's whole learning
schedule (1,048,576 vectors, 8 stages x 10 rounds), and all 64 slices of workload 3.  Same bars
as tests/test_gpu_parity.py; the oracle checks seeded rows one by one."""
import time

import numpy as np
import pytest

import oracle
from paper_2410_15704_amd import synth
from test_gpu_parity import _b, _frob_rel, _torch, _codebooks_from_samples, check_decode, check_encode

pytestmark = pytest.mark.gpu


def _say(capsys, msg):
    """A progress line that is not held back until the test ends."""
    with capsys.disabled():
        print("  [%s] %s" % (time.strftime("%H:%M:%S"), msg), flush=True)


# ------------------------------------------------------------------------- encode, K > 2048
@pytest.mark.parametrize("case", [
    # N, d, depth, K, dtype: vectors / 1024 = chunks; more than 256 chunks make workgroups walk on
    (2304, 4096, 8, 4096, "fp16"),    # 288 chunks, two pieces of 2048 codewords (workload 5's shape)
    (10240, 1024, 3, 2304, "bf16"),   # 320 chunks, a whole piece and one of 256 codewords
    (5000, 2048, 2, 6144, "fp32"),    # 313 chunks (the last one ragged), three pieces
])
def test_encode_large_codebook_persistent_workgroups(gpu_device, case):
    """A codebook that LDS does not hold is swept in pieces with workgroup barriers; here every
    workgroup also carries on from one chunk of vectors to the next."""
    N, d, depth, K, dtype = case
    if dtype == "fp16":
        X, _ = synth.heavy_tailed_keys(rows=slice(0, N))
    else:
        X = synth.gaussian_rows(N, d, seed=N + K, dtype=dtype, outliers=d // 50)
    Xw_head = synth.widen(X[:512], dtype)
    C = _codebooks_from_samples(Xw_head, 32, oracle.STRIDED, depth, K, seed=K)
    rows = np.sort(np.random.Generator(np.random.PCG64(K)).choice(N, 96, replace=False))
    rows[0], rows[-1] = 0, N - 1
    r = check_encode(X, dtype, d, 32, depth, K, oracle.STRIDED, C, sample_rows=rows)
    print("K = %d, %d chunks:" % (K, (N * (d // 32) + 1023) // 1024), r)


# ------------------------------------------------------------------------- workload 5
def test_long_context_full_size(gpu_device, capsys):
    """Workload 5 at full size: 131072 rows x 4096 channels fp16, strided groups (128 per row),
    depth 8, K = 4096: 16,777,216 group vectors = 16384 chunks, 64 per workgroup.  Encode, then
    decode after 1..8 stages.  The oracle checks 4096 seeded rows (first and last included): codes,
    near-tie proof, std, residual, decode, and the reconstruction error per depth to 1e-3."""
    torch, b = _torch(), _b()
    N, d, depth, K = 131072, 4096, 8, 4096
    Xh, _ = synth.heavy_tailed_keys()
    _say(capsys, "workload 5: input drawn")
    C = _codebooks_from_samples(synth.widen(Xh[:256], "fp16"), 32, oracle.STRIDED, depth, K, seed=5)
    rows = np.sort(np.random.Generator(np.random.PCG64(505)).choice(N, 4096, replace=False))
    rows[0], rows[-1] = 0, N - 1
    r = check_encode(Xh, "fp16", d, 32, depth, K, oracle.STRIDED, C, sample_rows=rows,
                     std_dtype="fp16", keep=True)
    q, codes, std, dX, ref = r["q"], r["codes"], r["std"], r["dX"], r["ref"]
    _say(capsys, "workload 5: encode checked on 4096 rows: %d of %d codes differ" %
         (r["mismatch"], r["entries"]))
    # decode after 1..8 stages (fp32 output of this quantizer): sampled rows against the oracle's
    # decode of the ORACLE's codes; all rows for the report
    rt = torch.from_numpy(rows).cuda()
    Xs = synth.widen(Xh[rows], "fp16")
    C64 = C.astype(np.float64)
    out = torch.empty((N, d), dtype=torch.float32, device="cuda")
    std64 = std[rt].float().cpu().numpy().astype(np.float64)  # the std the decode is handed
    mse_g, mse_o, mse_all = [], [], []
    for k in range(1, depth + 1):
        q.decode(codes, std, depth_used=k, out=out)
        got = out[rt].cpu().numpy().astype(np.float64)
        mse_g.append(np.mean((Xs - got) ** 2))
        want = oracle.decode(ref["codes"], std64, C64, d, oracle.STRIDED, depth_used=k)
        mse_o.append(np.mean((Xs - want) ** 2))
        acc = 0.0
        for a in range(0, N, 16384):
            acc += float(((dX[a:a + 16384].float() - out[a:a + 16384]) ** 2).sum(dtype=torch.float64))
        mse_all.append(acc / (N * d))
    q.close()
    _say(capsys, "workload 5 MSE per depth, all rows:     %s" % np.round(mse_all, 5).tolist())
    _say(capsys, "workload 5 MSE per depth, 4096 rows:    %s" % np.round(mse_g, 5).tolist())
    _say(capsys, "workload 5 MSE per depth, oracle codes: %s" % np.round(mse_o, 5).tolist())
    np.testing.assert_allclose(mse_g, mse_o, rtol=1e-3)
    np.testing.assert_allclose(mse_all, mse_o, rtol=0.05)  # all rows against the sample
    assert np.all(np.diff(mse_g) < 0)
    # decode parity proper (same codes to both sides), full N in the launch shape, both output types
    del out
    torch.cuda.empty_cache()
    for used in (8, 3):
        check_decode(None, None, "fp16", C, d, 32, oracle.STRIDED, depth_used=used, sample_rows=rows,
                     dev_codes=codes, dev_std=std)


# ------------------------------------------------------------------------- workload 4
W4 = dict(M=1048576, depth=8, K=2048, iters=10, decay=0.99, eps=1e-5)


def _w4_inputs():
    R = synth.gaussian_mixture(W4["M"])
    rng = np.random.Generator(np.random.PCG64(64))
    picks = [np.sort(rng.choice(W4["M"], W4["K"], replace=False)) for _ in range(W4["depth"])]
    return R, picks


def test_ema_full_schedule_every_pass_against_oracle(gpu_device, capsys):
    """Workload 4 as BASELINE names it: 1,048,576 mixture vectors, depth 8, K = 2048, stage by
    stage, 10 (assign, update) rounds per stage + the assignment that forms the residuals, decay
    0.99, eps 1e-5.  The schedule runs on the GPU through the library's entry points; EVERY one of
    its 88 passes is checked against the oracle from the state the GPU itself has reached (the
    rule the encode parity uses for later stages): the assignment under the GPU's current codebook
    (every differing code a near-tie of at most 1e-5 ||r||^2), then counts, sums and the new
    codebook given the GPU's codes (1e-5 relative), and the residuals passed to the next stage.
    Two free runs, one in fp32 and one in fp64, cannot be compared after 88 passes: see
    test_ema_full_schedule_free_running."""
    torch, b = _torch(), _b()
    M, depth, K, iters = W4["M"], W4["depth"], W4["K"], W4["iters"]
    decay, eps = np.float32(W4["decay"]), np.float32(W4["eps"])
    R0, picks = _w4_inputs()
    q = b.Quantizer(d=32, dhat=32, depth=depth, K=K, scale=0)
    C = torch.zeros((depth, K, 32), dtype=torch.float32, device="cuda")
    codes = torch.empty((M, 1, depth), dtype=torch.int16, device="cuda")
    R = torch.from_numpy(R0).cuda()
    flips_total, worst = 0, dict(cs=0.0, es=0.0, cb=0.0, tie=0.0)
    for s in range(depth):
        Rh = R.cpu().numpy().astype(np.float64)  # what enters stage s on the GPU
        C[s] = R.index_select(0, torch.from_numpy(picks[s]).cuda())
        q.set_codebooks(C)
        cs = torch.ones(K, dtype=torch.float32, device="cuda")
        es = C[s].clone()
        for it in range(iters + 1):
            Cs = q.get_codebooks()[s].cpu().numpy().astype(np.float64)
            last = it == iters
            _, _, res = q.encode(R, want_residual=last, stages=(s, s + 1), codes=codes)
            g = codes[:, 0, s].cpu().numpy().astype(np.int32)
            ref = oracle.encode(Rh, Cs[None], 32, scale=False, want_residual=last)
            o = ref["codes"].reshape(M)
            diff = np.nonzero(g != o)[0]
            flips_total += len(diff)
            if len(diff):  # the GPU's code must be as near as the oracle's, up to a near-tie
                dg = ((Rh[diff] - Cs[g[diff]]) ** 2).sum(axis=1)
                do = ((Rh[diff] - Cs[o[diff]]) ** 2).sum(axis=1)
                rel = (dg - do) / np.maximum((Rh[diff] ** 2).sum(axis=1), 1e-300)
                worst["tie"] = max(worst["tie"], float(rel.max()))
                assert rel.max() <= 1e-5
            assert len(diff) <= M * 1e-4
            if last:
                want = Rh - Cs[g]
                got = res.view(M, 32).cpu().numpy()
                assert np.abs(got - want).max() <= 1e-6 * np.abs(Rh).max()
                R = res.view(M, 32)
                break
            cs_h, es_h = cs.cpu().numpy().astype(np.float64), es.cpu().numpy().astype(np.float64)
            b.rvq_ema_update(q.ctx, s, R, codes.data_ptr() + 2 * s, depth, M, float(decay), float(eps), cs, es)
            cs_o, es_o, cb_o = oracle.ema_update(Rh, g, K, decay, eps, cs_h, es_h)
            e = (_frob_rel(cs.cpu().numpy(), cs_o), _frob_rel(es.cpu().numpy(), es_o),
                 _frob_rel(q.get_codebooks()[s].cpu().numpy(), cb_o))
            worst["cs"], worst["es"], worst["cb"] = max(worst["cs"], e[0]), max(worst["es"], e[1]), max(worst["cb"], e[2])
            assert max(e) <= 1e-5, (s, it, e)
        C = q.get_codebooks()
        _say(capsys, "workload 4: stage %d, 11 passes checked; codes that differ so far %d, largest "
             "errors so far %s" % (s, flips_total, {k: "%.1e" % v for k, v in worst.items()}))
    q.close()


def test_ema_full_schedule_free_running(gpu_device, capsys):
    """The same schedule run freely on both sides (train.ema_train_sequential against
    oracle.ema_train).  Learning a codebook is an iteration that amplifies differences: one vector
    whose two nearest codewords tie to 1e-7 goes one way in fp32 and the other way in fp64, the two
    codewords move, further vectors change sides in the next round, and the residuals handed to
    the later stages have little structure left to hold the partitions in place.  So the two runs
    agree closely in the first stage only, and what is compared over all stages is what the
    learning is for: the quantization error the learnt codebooks give, stage by stage.  The
    per-stage codebook differences and the share of final codes that differ are printed."""
    torch, b = _torch(), _b()
    from paper_2410_15704_amd import train
    M, depth, K, iters = W4["M"], W4["depth"], W4["K"], W4["iters"]
    R, picks = _w4_inputs()
    dR = torch.from_numpy(R).cuda()
    t0 = time.perf_counter()
    Cg = train.ema_train_sequential(dR, depth, K, iters, W4["decay"], W4["eps"], seed=0, picks=picks)
    torch.cuda.synchronize()
    _say(capsys, "workload 4 on the GPU: %.3f s for %d passes" % (time.perf_counter() - t0, depth * (iters + 1)))
    Co = oracle.ema_train(R.astype(np.float64), depth, K, iters, np.float32(W4["decay"]),
                          np.float32(W4["eps"]), picks, "sequential", progress=lambda m: _say(capsys, m))
    Cg = Cg.cpu().numpy()
    rels = [_frob_rel(Cg[s], Co[s]) for s in range(depth)]
    # each side quantizes the first 131072 vectors with its own codebooks (both by the oracle)
    head = R[:131072].astype(np.float64)
    og = oracle.encode(head, Cg.astype(np.float64), 32, scale=False)
    oo = oracle.encode(head, Co, 32, scale=False)
    flips = (og["codes"] != oo["codes"]).mean(axis=(0, 1))
    mse_g, mse_o = [], []
    for k in range(1, depth + 1):
        mse_g.append(np.mean((head - oracle.decode(og["codes"], np.ones(len(head)), Cg.astype(np.float64),
                                                   32, depth_used=k)) ** 2))
        mse_o.append(np.mean((head - oracle.decode(oo["codes"], np.ones(len(head)), Co, 32,
                                                   depth_used=k)) ** 2))
    _say(capsys, "workload 4 free run, codebook difference per stage: %s" % ["%.1e" % x for x in rels])
    _say(capsys, "workload 4 free run, share of codes that differ:    %s" % ["%.1e" % x for x in flips])
    _say(capsys, "workload 4 error per depth, GPU-learnt codebooks:    %s" % np.round(mse_g, 6).tolist())
    _say(capsys, "workload 4 error per depth, oracle-learnt codebooks: %s" % np.round(mse_o, 6).tolist())
    assert rels[0] <= 1e-3
    np.testing.assert_allclose(mse_g, mse_o, rtol=1e-2)
    assert np.all(np.diff(mse_g) < 0)


# ------------------------------------------------------------------------- workload 3
def test_decode_all_64_slices_sampled_oracle(gpu_device, capsys):
    """Workload 3 as the benchmark streams it: 64 (layer, key / value) slices of 524288 tokens x
    1024 channels, each with its own codebook set, even slices strided and odd ones contiguous,
    int16 codes drawn on the device, fp16 std.  Slice 0 is checked in full, every other slice on
    4096 seeded rows, in both output types."""
    torch = _torch()
    S, T = 64, 16 * 32768
    Cs = synth.decode_codebooks(S)
    std_all = synth.decode_std_fp16(S * T).reshape(S, T)
    worst = 0.0
    for s in range(S):
        grouping = oracle.STRIDED if s % 2 == 0 else oracle.CONTIGUOUS
        codes = synth.uniform_codes_device(T, 32, 8, 2048, "cuda", extra=100 + s)
        std = torch.from_numpy(std_all[s]).cuda()
        if s == 0:
            for a in range(0, T, 65536):  # in full, 65536 rows at a time
                r = check_decode(None, None, "fp16", Cs[s], 1024, 32, grouping,
                                 sample_rows=np.arange(a, a + 65536), dev_codes=codes, dev_std=std)
                worst = max(worst, r["max_rel"])
        else:
            rows = np.sort(np.random.Generator(np.random.PCG64(3000 + s)).choice(T, 4096, replace=False))
            rows[0], rows[-1] = 0, T - 1
            r = check_decode(None, None, "fp16", Cs[s], 1024, 32, grouping, sample_rows=rows,
                             dev_codes=codes, dev_std=std)
            worst = max(worst, r["max_rel"])
        del codes, std
        if s % 8 == 7:
            _say(capsys, "workload 3: slices 0..%d checked, largest row error %.2e" % (s, worst))
    torch.cuda.empty_cache()


# ------------------------------------------------------------------------- EMA histogram widths
@pytest.mark.parametrize("M,K", [
    (50000, 1024),    # channel slices of 16
    (120000, 4096),   # slices of 4 (workload 5's codebook size)
    (90000, 6000),    # slices of 2
    (90000, 8192),    # slices of 1
    (20000, 256),     # one slice of 32
])
def test_ema_update_every_slice_width(gpu_device, M, K):
    """rvq_ema_update cuts the 32 channels into slices so that K x slice sums fit LDS; every slice
    width it can choose, against the oracle with the same codes."""
    torch, b = _torch(), _b()
    dhat = 32
    rng = np.random.Generator(np.random.PCG64(M + K))
    R = synth.gaussian_mixture(M, dhat, n_comp=16, index=4 + K % 7)
    codes = rng.integers(0, K, size=M).astype(np.int16)
    codes[:4] = [0, K - 1, K - 1, 1]
    C0 = rng.standard_normal((K, dhat)).astype(np.float32)
    cs0 = (0.5 + rng.random(K)).astype(np.float32)
    es0 = (C0 * cs0[:, None]).astype(np.float32)
    q = b.Quantizer(d=dhat, dhat=dhat, depth=1, K=K, scale=0)
    q.set_codebooks(torch.from_numpy(C0[None].copy()).cuda())
    d_cs, d_es = torch.from_numpy(cs0.copy()).cuda(), torch.from_numpy(es0.copy()).cuda()
    q.ema_update(0, torch.from_numpy(R).cuda(), torch.from_numpy(codes).cuda(), d_cs, d_es,
                 decay=0.9, eps=1e-5)
    cs, es, cb = oracle.ema_update(R.astype(np.float64), codes.astype(np.int32), K, np.float32(0.9),
                                   np.float32(1e-5), cs0.astype(np.float64), es0.astype(np.float64))
    assert _frob_rel(d_cs.cpu().numpy(), cs) <= 1e-5
    assert _frob_rel(d_es.cpu().numpy(), es) <= 1e-5
    assert _frob_rel(q.get_codebooks().cpu().numpy()[0], cb) <= 1e-5
    q.close()


# ------------------------------------------------------------------------- row strides
@pytest.mark.parametrize("case", [
    # N, d, depth, K, grouping, dtype, ldx
    (300, 256, 4, 128, oracle.STRIDED, "fp32", 264),      # rows stay 16-byte aligned
    (300, 256, 4, 128, oracle.CONTIGUOUS, "bf16", 264),
    (300, 256, 4, 128, oracle.STRIDED, "fp16", 259),      # rows off every vector boundary
    (2100, 1024, 8, 2048, oracle.STRIDED, "bf16", 1040),  # the benchmark's shape, padded rows
    (64, 48, 3, 20, oracle.CONTIGUOUS, "fp32", 50),       # the generic path (dhat 8)
])
def test_encode_row_stride(gpu_device, case):
    N, d, depth, K, grouping, dtype, ldx = case
    dhat = 8 if d == 48 else 32
    X = synth.gaussian_rows(N, d, seed=N + ldx, dtype=dtype, outliers=2)
    C = _codebooks_from_samples(synth.widen(X, dtype), dhat, grouping, depth, K, seed=ldx)
    rows = None if N <= 300 else np.arange(0, N, 7)
    check_encode(X, dtype, d, dhat, depth, K, grouping, C, ldx=ldx, sample_rows=rows)


@pytest.mark.parametrize("case", [
    # N, d, dhat, depth, K, grouping, ldo, packed
    (700, 1024, 32, 8, 2048, oracle.CONTIGUOUS, 1032, False),  # row-gather kernel, 16-byte rows kept
    (700, 1024, 32, 8, 2048, oracle.STRIDED, 1032, False),
    (700, 1024, 32, 8, 2048, oracle.STRIDED, 1028, True),      # 8-byte rows only
    (16500, 1024, 32, 8, 2048, oracle.STRIDED, 1028, False),   # enough rows for the LDS kernel
    (16500, 1024, 32, 8, 2048, oracle.STRIDED, 1040, True),
    (300, 256, 32, 5, 100, oracle.STRIDED, 261, False),        # rows off every boundary: generic kernel
    (300, 256, 32, 5, 100, oracle.CONTIGUOUS, 257, False),
    (120, 48, 8, 3, 20, oracle.STRIDED, 64, False),
])
def test_decode_row_stride(gpu_device, case):
    """Decode into a buffer whose rows are longer than d: same values as the decode into a dense
    buffer, bit for bit, in both output types, and nothing written beyond channel d of a row."""
    torch, b = _torch(), _b()
    N, d, dhat, depth, K, grouping, ldo, packed = case
    G = d // dhat
    rng = np.random.Generator(np.random.PCG64(N + ldo))
    codes = torch.from_numpy(rng.integers(0, K, size=(N, G, depth)).astype(np.int16)).cuda()
    std = torch.from_numpy(np.exp(0.3 * rng.standard_normal(N)).astype(np.float16)).cuda()
    C = (rng.standard_normal((depth, K, dhat)) * (0.6 ** np.arange(depth))[:, None, None]).astype(np.float32)
    for odt, tdt in ((b.F16, torch.float16), (b.F32, torch.float32)):
        q = b.Quantizer(d=d, dhat=dhat, depth=depth, K=K, grouping=grouping, out_dtype=odt, std_dtype=b.F16)
        q.set_codebooks(torch.from_numpy(C).cuda())
        dense = q.decode(codes, std)
        wide = torch.full((N, ldo), -3.0, dtype=tdt, device="cuda")
        view = wide[:, :d]
        if packed:
            q.decode_packed(q.pack(codes), std, out=view)
        else:
            q.decode(codes, std, out=view)
        torch.cuda.synchronize()
        assert torch.equal(view, dense)
        assert bool((wide[:, d:] == -3.0).all())
        q.close()
    rows = np.arange(0, N, max(1, N // 300))
    check_decode(codes.cpu().numpy(), std.cpu().numpy(), "fp16", C, d, dhat, grouping, sample_rows=rows)


# ------------------------------------------------------------------------- boundary
def test_enqueue_calls_neither_allocate_nor_synchronize(gpu_device):
    """rvq_encode with growing N and the first rvq_ema_update of a context, on a stream of their
    own that is still busy: the calls return while work enqueued before them is still running
    (an event recorded before them is still pending afterwards), and rows beyond the reserved
    workspace are refused until rvq_reserve has been called."""
    torch, b = _torch(), _b()
    d, depth, K = 1024, 8, 2048
    Xb, _ = synth.llama_key(32768, d)
    dX = torch.from_numpy(Xb.view(np.int16)).cuda().view(torch.bfloat16)
    C = torch.randn((depth, K, 32), device="cuda") * 0.5
    q = b.Quantizer(d=d, dhat=32, depth=depth, K=K, grouping=b.STRIDED, in_dtype=b.BF16)
    q.set_codebooks(C)
    codes = torch.empty((32768, 32, depth), dtype=torch.int16, device="cuda")
    std = torch.empty(32768, dtype=torch.float16, device="cuda")
    Z = torch.randn((1 << 20, 32), device="cuda")
    cs, es = torch.ones(K, device="cuda"), C[0].clone()
    qe = b.Quantizer(d=32, dhat=32, depth=depth, K=K, scale=0)
    qe.set_codebooks(C)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    ev = torch.cuda.Event()
    with torch.cuda.stream(s):
        for _ in range(12):  # some 20 ms of work ahead of the calls under test
            b.rvq_encode(q.ctx, dX, 32768, d, 0, depth, codes, std, None)
        ev.record(s)
        for n in (1024, 4096, 32768):  # growing N
            b.rvq_encode(q.ctx, dX, n, d, 0, depth, codes, std, None)
        b.rvq_ema_update(qe.ctx, 0, Z, codes, depth, 1 << 20, 0.99, 1e-5, cs, es)
        pending = not ev.query()
    torch.cuda.synchronize()
    assert pending, "an enqueue call waited for the device"
    assert b.rvq_check_kernels(q.ctx) == 0
    # the workspace limit
    assert b.rvq_reserved_rows(q.ctx) == b.DEFAULT_ROWS
    assert b.rvq_reserved_rows(qe.ctx) > 1 << 60  # rows that are not scaled need no workspace
    big = b.DEFAULT_ROWS + 1
    xb = torch.zeros((big, d), dtype=torch.bfloat16, device="cuda")
    cb = torch.empty((big, 32, depth), dtype=torch.int16, device="cuda")
    sb = torch.empty(big, dtype=torch.float16, device="cuda")
    rc = b.lib.rvq_encode(q.ctx, xb.data_ptr(), big, d, 0, depth, cb.data_ptr(), sb.data_ptr(), None,
                          torch.cuda.current_stream().cuda_stream)
    assert rc == b.RVQ_EWORKSPACE
    assert "rvq_reserve" in b.rvq_strerror(rc)
    b.rvq_reserve(q.ctx, big)
    assert b.rvq_reserved_rows(q.ctx) == big
    b.rvq_encode(q.ctx, xb, big, d, 0, depth, cb, sb, None)
    torch.cuda.synchronize()
    assert b.lib.rvq_reserve(q.ctx, -1) == b.RVQ_EINVAL
    q.close()
    qe.close()


def test_bounded_wait_reports_instead_of_hanging(gpu_device):
    """The wavefronts of the encode kernel wait for each other through counters in LDS.  With the
    bound on those waits set to zero polls every wait that is not already satisfied gives up: the
    kernel must still run to its end, the context must report RVQ_EKERNEL once, and with the
    default bound the same context must encode correctly again."""
    torch, b = _torch(), _b()
    N, d, depth, K = 2048, 1024, 8, 2048
    X, _ = synth.llama_key(N, d)
    C = _codebooks_from_samples(synth.widen(X[:256], "bf16"), 32, oracle.STRIDED, depth, K, seed=9)
    q = b.Quantizer(d=d, dhat=32, depth=depth, K=K, grouping=b.STRIDED, in_dtype=b.BF16, std_dtype=b.F32)
    q.set_codebooks(torch.from_numpy(C).cuda())
    dX = torch.from_numpy(X.view(np.int16)).cuda().view(torch.bfloat16)
    good, _, _ = q.encode(dX)
    assert b.rvq_check_kernels(q.ctx, check=False) == 0
    b.rvq_debug_set_wait_polls(q.ctx, 0)
    junk, _, _ = q.encode(dX)
    torch.cuda.synchronize()
    assert int(junk.min()) >= 0 and int(junk.max()) < K  # still codes, whatever their value
    assert b.rvq_check_kernels(q.ctx, check=False) == b.RVQ_EKERNEL
    assert b.rvq_check_kernels(q.ctx, check=False) == 0  # reported once
    b.rvq_debug_set_wait_polls(q.ctx, 1 << 22)
    again, _, _ = q.encode(dX)
    assert torch.equal(again, good)
    assert b.rvq_check_kernels(q.ctx, check=False) == 0
    assert b.lib.rvq_debug_set_wait_polls(q.ctx, -1) == b.RVQ_EINVAL
    q.close()


# ------------------------------------------------------------------------- non-finite inputs
@pytest.mark.parametrize("case", [
    # d, dhat, K, depth, grouping: the matrix-core path (dhat 32) and the plain scan (dhat 16)
    (256, 32, 300, 4, oracle.STRIDED),
    (256, 32, 64, 3, oracle.CONTIGUOUS),
    (64, 16, 50, 3, oracle.CONTIGUOUS),
])
def test_rows_with_nan_or_infinity_leave_the_other_rows_alone(gpu_device, case):
    """The boundary asks for finite inputs and promises, for a row that has a NaN or an infinity,
    codes inside [0, K), no access out of bounds and no effect on any other row.  Rows 3, 7, 100,
    200 and the last one are poisoned; every other row must get exactly the codes and the std
    of a run without the poison."""
    torch, b = _torch(), _b()
    d, dhat, K, depth, grouping = case
    N = 1300  # more than one chunk of 1024 group vectors per workgroup and a ragged tail
    rng = np.random.Generator(np.random.PCG64(d + K))
    X = rng.standard_normal((N, d)).astype(np.float32)
    C = (rng.standard_normal((depth, K, dhat)) * (0.7 ** np.arange(depth))[:, None, None]).astype(np.float32)
    bad = X.copy()
    bad[3, 5] = np.nan
    bad[7, 0] = np.inf
    bad[100, d - 1] = -np.inf
    bad[200, :] = np.nan
    bad[N - 1, 17] = np.inf
    bad[N - 1, 18] = np.nan
    poisoned = np.array([3, 7, 100, 200, N - 1])
    clean_rows = np.setdiff1d(np.arange(N), poisoned)
    q = b.Quantizer(d=d, dhat=dhat, depth=depth, K=K, grouping=grouping, in_dtype=b.F32, std_dtype=b.F32)
    q.set_codebooks(torch.from_numpy(C).cuda())
    c0, s0, _ = q.encode(torch.from_numpy(X).cuda())
    c1, s1, _ = q.encode(torch.from_numpy(bad).cuda())
    torch.cuda.synchronize()
    assert b.rvq_check_kernels(q.ctx) == 0
    # and decoding whatever codes came out stays in bounds too
    out = q.decode(c1, s1)
    torch.cuda.synchronize()
    h0, h1 = c0.cpu().numpy(), c1.cpu().numpy()
    assert h1.min() >= 0 and h1.max() < K
    assert np.array_equal(h1[clean_rows], h0[clean_rows])
    assert np.array_equal(s1.cpu().numpy()[clean_rows], s0.cpu().numpy()[clean_rows])
    assert np.isfinite(out.float().cpu().numpy()[clean_rows]).all()
    q.close()


# ------------------------------------------------------------------------- the ceiling probes
def test_gather_rate_probes_return_plausible_rates(gpu_device):
    """rvq_probe_gather_rates measures what this GPU delivers for the decode kernels' gathers; bench.py
    prices the decode ceilings with it.  The three rates must be positive and ordered as the
    hardware orders them: consecutive LDS reads faster than random ones, and all of them above the
    HBM rate that the decode paths are compared with."""
    b = _b()
    r = b.rvq_probe_gather_rates()
    assert set(r) == {"lds_random_GBs", "lds_consecutive_GBs", "l2_rows_random_GBs"}
    assert r["lds_consecutive_GBs"] > r["lds_random_GBs"] > 8000.0
    assert r["l2_rows_random_GBs"] > 8000.0
    assert r["lds_consecutive_GBs"] < 400000.0  # (256 CUs x 128 B/clk x 2.4 GHz = 78,600)
