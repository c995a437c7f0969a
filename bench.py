#!/usr/bin/env python3
"""Benchmark of the RVQ hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-decode-stream] [--no-cpu]

A step is one pass of the whole hot path over one batch of workload 2 (Llama-3-8B-like key
projection: N=32768 rows x 1024 channels, bf16, strided groups of 32, depth 8, K=2048):
    rvq_encode   per-row std, grouping, 8 stages of distance + argmin + residual update
    rvq_decode   gather + sum + rescale of the codes just produced, fp16 out
    rvq_ema_update  one moving-average update of codebook 0 from the batch's 1,048,576 scaled
                 group vectors and their stage-0 codes (scatter + blend)
Inputs are resident in HBM before the timed region.  One JSON line is printed:
value = group vectors per second through the whole step; `roofline` describes the encode kernel
(the dominant one) against the dense fp16/bf16 matrix-core peak; `decode_stream` is the decode
kernel alone over workload 3 (64 slices of 524288 tokens, 85.97 GB of traffic) against the HBM
peak; `cpu_baseline` is the fp64 oracle timed on the host cores on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_16BIT_TFLOPS = 2500.0  # MI355X dense bf16 / fp16 matrix-core peak
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E
# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of `--profile encode` and
# `--profile decode`, scaled by the readings of a plain 1 GiB copy: FETCH_SIZE counts 2 KiB units,
# WRITE_SIZE 1 KiB units (the readings are in profiles/rvq_encode_workload2.txt and
# profiles/rvq_decode_workload3_slice.txt)
TRAFFIC_ENCODE_W2 = 1.1563e5 * 2048 + 1.2123e5 * 1024            # encode_screen_kernel, workload 2
TRAFFIC_DECODE_SLICE = 0.5 * ((1.4005e5 + 1.4058e5) * 2048) + 1.0486e6 * 1024  # mean of both kernels

W2 = dict(N=32768, d=1024, dhat=32, depth=8, K=2048)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-decode-stream", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-extra-workloads", action="store_true",
                    help="skip the workload 4 and workload 5 legs")
    ap.add_argument("--decode-slices", type=int, default=64)
    ap.add_argument("--cpu-rows", type=int, default=32768)
    ap.add_argument("--encode-path", type=int, default=0)
    ap.add_argument("--profile", choices=["encode", "decode", "ema", "attn", "append", "copy"], default=None,
                    help="run only one kernel a few times (for rocprofv3 runs; prints no JSON)")
    return ap.parse_args()


class EventTimer:
    """HIP events on torch's current stream (the stream every library call is enqueued on)."""

    def __init__(self):
        import torch
        self.torch = torch
        self.pairs = {}

    def record(self, name, fn):
        a = self.torch.cuda.Event(enable_timing=True)
        b = self.torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        self.pairs.setdefault(name, []).append((a, b))

    def mean_ms(self, name):
        p = self.pairs.get(name, [])
        return sum(a.elapsed_time(b) for a, b in p) / max(1, len(p))


def run_steps(args):
    import numpy as np
    import torch

    from paper_2410_15704_amd import binding as b
    from paper_2410_15704_amd import synth, train

    N, d, dhat, depth, K = (W2[k] for k in ("N", "d", "dhat", "depth", "K"))
    G = d // dhat
    V = N * G
    Xb, _ = synth.llama_key(N, d)
    dX = torch.from_numpy(Xb.view(np.int16)).cuda().view(torch.bfloat16)
    # sample-initialised codebooks from the first 2048 rows, built by the library itself
    Zhead = train.scaled_groups(dX[:2048], d=d, dhat=dhat, grouping=b.STRIDED, in_dtype=b.BF16)
    C = train.sample_init_codebooks(Zhead, depth, K, seed=synth.BASE_SEED + 2)
    del Zhead
    Z = train.scaled_groups(dX, d=d, dhat=dhat, grouping=b.STRIDED, in_dtype=b.BF16)  # EMA input

    q = b.Quantizer(d=d, dhat=dhat, depth=depth, K=K, grouping=b.STRIDED, in_dtype=b.BF16,
                    out_dtype=b.F16, std_dtype=b.F16, encode_path=args.encode_path)
    q.set_codebooks(C)
    codes = torch.empty((N, G, depth), dtype=torch.int16, device="cuda")
    std = torch.empty((N,), dtype=torch.float16, device="cuda")
    out = torch.empty((N, d), dtype=torch.float16, device="cuda")
    cs = torch.ones(K, dtype=torch.float32, device="cuda")
    es = C[0].clone()

    def enc():
        b.rvq_encode(q.ctx, dX, N, d, 0, depth, codes, std, None)

    def dec():
        b.rvq_decode(q.ctx, codes, std, N, depth, out, d)

    def ema():
        b.rvq_ema_update(q.ctx, 0, Z, codes, depth, V, 0.99, 1e-5, cs, es)  # code of vector v: codes[v * depth]

    for _ in range(args.warmup):
        enc(); dec(); ema()
    torch.cuda.synchronize()
    tm = EventTimer()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        tm.record("encode", enc)
        tm.record("decode", dec)
        tm.record("ema", ema)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    enc_ms, dec_ms, ema_ms = tm.mean_ms("encode"), tm.mean_ms("decode"), tm.mean_ms("ema")
    flops = 2.0 * dhat * K * depth * V  # 2 * dhat * K flop per vector and stage
    enc_tflops = flops / (enc_ms * 1e-3) / 1e12
    dec_bytes = N * (G * depth * 2 + 2 + d * 2)
    ema_bytes = V * (dhat * 4 + 2)
    res = dict(
        ms_per_step=ms_step, vec_per_step=V,
        breakdown=dict(
            encode_ms=enc_ms, decode_ms=dec_ms, ema_update_ms=ema_ms,
            encode_Mvec_s=V / (enc_ms * 1e-3) / 1e6,
            encode_tflops=enc_tflops,
            encode_frac_of_mfma_peak=enc_tflops / PEAK_MFMA_16BIT_TFLOPS,
            decode_GBs=dec_bytes / (dec_ms * 1e-3) / 1e9,
            decode_frac_of_hbm_peak=dec_bytes / (dec_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
            ema_GBs=ema_bytes / (ema_ms * 1e-3) / 1e9,
        ),
        roofline=dict(bound="mfma", achieved=enc_tflops, peak=PEAK_MFMA_16BIT_TFLOPS,
                      unit="TFLOP/s", frac=enc_tflops / PEAK_MFMA_16BIT_TFLOPS,
                      traffic=TRAFFIC_ENCODE_W2,
                      kernel="rvq_encode (all 8 stages, one launch per call)",
                      flops_per_launch=flops, avg_launch_ms=enc_ms),
    )
    q.close()
    del dX, Z, codes, std, out
    torch.cuda.empty_cache()
    return res


def run_decode_stream(args):
    """Workload 3: decode-time reconstruction of a whole KV cache, 64 (layer, K/V) slices of
    16 x 32768 tokens x 1024 channels, int16 codes + fp16 std -> fp16."""
    import torch

    from paper_2410_15704_amd import binding as b
    from paper_2410_15704_amd import synth

    S = args.decode_slices
    T, d, G, depth, K = 16 * 32768, 1024, 32, 8, 2048
    need = S * T * (G * depth * 2 + 2 + d * 2) + (2 << 30)
    free, _ = torch.cuda.mem_get_info()
    if need > free:
        S = max(1, int((free - (2 << 30)) // (T * (G * depth * 2 + 2 + d * 2))))
    Cs = torch.from_numpy(synth.decode_codebooks(S)).cuda()
    qs = []
    for s in range(S):
        q = b.Quantizer(d=d, dhat=32, depth=depth, K=K, out_dtype=b.F16, std_dtype=b.F16,
                        grouping=b.STRIDED if s % 2 == 0 else b.CONTIGUOUS)
        q.set_codebooks(Cs[s])
        qs.append(q)
    codes = [synth.uniform_codes_device(T, G, depth, K, "cuda", extra=100 + s) for s in range(S)]
    std = torch.from_numpy(synth.decode_std_fp16(S * T)).cuda().view(S, T)
    out = torch.empty((S, T, d), dtype=torch.float16, device="cuda")

    def one_pass():
        for s in range(S):
            b.rvq_decode(qs[s].ctx, codes[s], std[s], T, depth, out[s], d)

    one_pass()
    torch.cuda.synchronize()
    reps = 3
    a = torch.cuda.Event(enable_timing=True)
    z = torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        one_pass()
    z.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(z) / reps
    nbytes = S * T * (G * depth * 2 + 2 + d * 2)
    gbs = nbytes / (ms * 1e-3) / 1e9
    # the same decode from 11-bit packed records (352 instead of 512 bytes of codes per token), on
    # one strided and one contiguous slice, next to the int16 decode of that slice repeated in the
    # same way (a slice that is decoded over and over keeps part of its codes in the Infinity
    # Cache, so these two compare with each other, not with the 64-slice stream above)
    packed = {}
    # rotary tables (inputs of rvq_decode_rope): 8 heads of 128 channels, positions 0..32767
    hd = 128
    ang = (torch.arange(T, device="cuda") % 32768).double()[:, None] * \
        (10000.0 ** (-2.0 * torch.arange(hd // 2, device="cuda").double() / hd))[None, :]
    dcos, dsin = torch.cos(ang).float(), torch.sin(ang).float()
    del ang
    for s_ in range(min(S, 2)):
        pk = qs[s_].pack(codes[s_])
        res = {}
        for name, fn in (("int16", lambda: b.rvq_decode(qs[s_].ctx, codes[s_], std[s_], T, depth, out[s_], d)),
                         ("packed", lambda: b.rvq_decode_packed(qs[s_].ctx, pk, std[s_], T, depth, out[s_], d)),
                         ("rope", lambda: b.rvq_decode_rope(qs[s_].ctx, codes[s_], std[s_], T, depth, dcos,
                                                            dsin, hd, out[s_], d))):
            fn()
            torch.cuda.synchronize()
            a.record()
            for _ in range(5):
                fn()
            z.record()
            torch.cuda.synchronize()
            res[name + "_ms_per_slice"] = a.elapsed_time(z) / 5
        pbytes = T * (pk.shape[1] * pk.shape[2] + 2 + d * 2)
        res["packed_bytes_per_slice"] = pbytes
        res["packed_GBs"] = pbytes / (res["packed_ms_per_slice"] * 1e-3) / 1e9
        res["packed_tokens_per_s"] = T / (res["packed_ms_per_slice"] * 1e-3)
        packed["strided" if s_ % 2 == 0 else "contiguous"] = res
        del pk
    del dcos, dsin
    for q in qs:
        q.close()
    # What bounds the decode is not HBM but the on-chip gather: 32 groups x 8 stages x 128 bytes of
    # fp32 codeword rows = 32 KiB per token against 2562 bytes of HBM traffic.  The library's probes
    # measure the rate at which this GPU gathers in the two kernels' access shapes; divided by the
    # 32 KiB per token and multiplied by the 2562 HBM bytes per token they give the decode rate at
    # which the gathers alone would saturate, to compare with what each kernel reaches.
    pr = b.rvq_probe_gather_rates()
    gather_bytes = G * depth * 32 * 4
    row_bytes = G * depth * 2 + 2 + d * 2
    slice_bytes = T * row_bytes
    ceil_lds = pr["lds_random_GBs"] / gather_bytes * row_bytes
    ceil_lds_free = pr["lds_consecutive_GBs"] / gather_bytes * row_bytes
    ceil_l2 = pr["l2_rows_random_GBs"] / gather_bytes * row_bytes
    ceiling = dict(gather_bytes_per_token=gather_bytes, hbm_bytes_per_token=row_bytes, probes_GBs=pr,
                   lds_kernel=dict(grouping="strided", bound="LDS reads at random addresses",
                                   ceiling_GBs=ceil_lds, ceiling_without_bank_conflicts_GBs=ceil_lds_free),
                   row_gather_kernel=dict(grouping="contiguous", bound="L2 row gathers", ceiling_GBs=ceil_l2))
    for key, name in (("lds_kernel", "strided"), ("row_gather_kernel", "contiguous")):
        if name in packed:
            gb = slice_bytes / (packed[name]["int16_ms_per_slice"] * 1e-3) / 1e9
            ceiling[key].update(achieved_GBs=gb, frac_of_ceiling=gb / ceiling[key]["ceiling_GBs"],
                                frac_of_hbm_peak=gb / PEAK_HBM_GBS)
    return dict(workload="decode-time reconstruction, %d slices x 524288 tokens x 1024 ch" % S,
                slices=S, ms_per_pass=ms, bytes_per_pass=nbytes, tokens_per_s=S * T / (ms * 1e-3),
                packed_codes_and_rope=packed, ceiling=ceiling,
                roofline=dict(bound="hbm", achieved=gbs, peak=PEAK_HBM_GBS, unit="GB/s",
                              frac=gbs / PEAK_HBM_GBS, traffic=TRAFFIC_DECODE_SLICE,
                              kernel="rvq_decode", bytes_per_launch=nbytes / S,
                              avg_launch_ms=ms / S))


def run_workload5(args):
    """Workload 5 (long-context MHA): N = 131072 rows x 4096 channels fp16, strided groups (128 per
    row), depth 8, K = 4096: encode, decode, reconstruction error after 1..8 stages.  The rows are
    drawn on the device (torch's seeded generator) with the workload's recipe, N(0,1) times a
    per-channel scale min(100, Pareto(1.5))."""
    import numpy as np
    import torch

    from paper_2410_15704_amd import binding as b
    from paper_2410_15704_amd import synth, train

    N, d, dhat, depth, K = 131072, 4096, 32, 8, 4096
    G, V = d // dhat, N * (d // dhat)
    _, sigma = synth.heavy_tailed_keys(rows=slice(0, 1))  # the workload's seeded channel scales
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.BASE_SEED + 5)
    dX = torch.empty((N, d), dtype=torch.float16, device="cuda")
    sg = torch.from_numpy(sigma).cuda()
    for a in range(0, N, 16384):
        dX[a:a + 16384] = (torch.randn((16384, d), device="cuda", generator=gen) * sg).half()
    Zhead = train.scaled_groups(dX[:512], d=d, dhat=dhat, grouping=b.STRIDED, in_dtype=b.F16)
    C = train.sample_init_codebooks(Zhead, depth, K, seed=synth.BASE_SEED + 5)
    del Zhead
    q = b.Quantizer(d=d, dhat=dhat, depth=depth, K=K, grouping=b.STRIDED, in_dtype=b.F16,
                    out_dtype=b.F16, std_dtype=b.F16)
    q.set_codebooks(C)
    codes = torch.empty((N, G, depth), dtype=torch.int16, device="cuda")
    std = torch.empty((N,), dtype=torch.float16, device="cuda")
    out = torch.empty((N, d), dtype=torch.float16, device="cuda")
    a, z = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        z.record()
        torch.cuda.synchronize()
        return a.elapsed_time(z) / reps

    enc_ms = timed(lambda: b.rvq_encode(q.ctx, dX, N, d, 0, depth, codes, std, None), 3)
    dec_ms = timed(lambda: b.rvq_decode(q.ctx, codes, std, N, depth, out, d), 5)
    mse = []
    for k in range(1, depth + 1):
        b.rvq_decode(q.ctx, codes, std, N, k, out, d)
        acc = 0.0
        for r0 in range(0, N, 16384):
            acc += float(((dX[r0:r0 + 16384].float() - out[r0:r0 + 16384].float()) ** 2).sum(dtype=torch.float64))
        mse.append(acc / (N * d))
    flops = 2.0 * dhat * K * depth * V
    dec_bytes = N * (G * depth * 2 + 2 + d * 2)
    q.close()
    return dict(workload="workload 5: N=131072 x 4096 ch fp16, strided, 128 groups, depth 8, K=4096",
                vectors=V, encode_ms=enc_ms, encode_Mvec_s=V / (enc_ms * 1e-3) / 1e6,
                encode_tflops=flops / (enc_ms * 1e-3) / 1e12,
                encode_frac_of_mfma_peak=flops / (enc_ms * 1e-3) / 1e12 / PEAK_MFMA_16BIT_TFLOPS,
                decode_ms=dec_ms, decode_GBs=dec_bytes / (dec_ms * 1e-3) / 1e9,
                decode_frac_of_hbm_peak=dec_bytes / (dec_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                mse_per_depth=mse, mean_square_of_input=float((dX[:16384].float() ** 2).mean()))


def run_append(args):
    """What a serving loop does per generated token: encode the few rows that were appended
    (1, 8, 64 rows of workload 2's shape; 2048 rows for a prefill chunk) and decode a short cache
    (1024 and 8192 rows).  Times
    per call in microseconds, stream time over 200 calls back to back (one kernel per encode of so
    few rows: std and search together)."""
    import numpy as np
    import torch

    from paper_2410_15704_amd import binding as b
    from paper_2410_15704_amd import synth, train

    d, dhat, depth, K = (W2[k] for k in ("d", "dhat", "depth", "K"))
    G = d // dhat
    Xb, _ = synth.llama_key(8192, d)
    dX = torch.from_numpy(Xb.view(np.int16)).cuda().view(torch.bfloat16)
    Zhead = train.scaled_groups(dX[:2048], d=d, dhat=dhat, grouping=b.STRIDED, in_dtype=b.BF16)
    C = train.sample_init_codebooks(Zhead, depth, K, seed=synth.BASE_SEED + 2)
    q = b.Quantizer(d=d, dhat=dhat, depth=depth, K=K, grouping=b.STRIDED, in_dtype=b.BF16,
                    out_dtype=b.F16, std_dtype=b.F16)
    q.set_codebooks(C)
    codes = torch.empty((8192, G, depth), dtype=torch.int16, device="cuda")
    std = torch.empty((8192,), dtype=torch.float16, device="cuda")
    out = torch.empty((8192, d), dtype=torch.float16, device="cuda")
    b.rvq_encode(q.ctx, dX, 8192, d, 0, depth, codes, std, None)
    a, z = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def us(fn, reps=200):
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        z.record()
        torch.cuda.synchronize()
        return a.elapsed_time(z) / reps * 1e3

    res = {}
    for n in (1, 8, 64, 2048):  # 2048: a prefill chunk (matrix-core kernel, one token per lane)
        res["encode_%d_rows_us" % n] = us(lambda: b.rvq_encode(q.ctx, dX, n, d, 0, depth, codes, std, None))
    for n in (1024, 8192):
        res["decode_%d_rows_us" % n] = us(lambda: b.rvq_decode(q.ctx, codes, std, n, depth, out, d))
    q.close()
    return res


def run_attn_decode(args):
    """Attention of one query position over a cache of codes (`rvq_attn_decode`): 131072 tokens x 8
    kv heads of 128 channels, 4 query heads per kv head, keys strided / values contiguous, depth
    8, K = 2048, seeded uniform codes.  Beside it the unfused route through the library's own
    decode calls (fp16 keys with the rotary embedding and fp16 values written out) - the attention
    that would then read them is not timed."""
    import torch

    from paper_2410_15704_amd import binding as b
    from paper_2410_15704_amd import synth

    N, Hkv, rep, depth, K, hd = 131072, 8, 4, 8, 2048, 128
    Hq, rows = Hkv * rep, N * Hkv
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.BASE_SEED + 6)
    Ck = torch.randn((depth, K, 32), device="cuda", generator=gen)
    Cv = torch.randn((depth, K, 32), device="cuda", generator=gen)
    kc = torch.randint(0, K, (rows, 4, depth), device="cuda", generator=gen, dtype=torch.int16)
    vc = torch.randint(0, K, (rows, 4, depth), device="cuda", generator=gen, dtype=torch.int16)
    ks = (torch.rand(rows, device="cuda", generator=gen) + 0.5).half()
    vs = (torch.rand(rows, device="cuda", generator=gen) + 0.5).half()
    qv = torch.randn((Hq, hd), device="cuda", generator=gen)
    ang = torch.rand((N, hd // 2), device="cuda", generator=gen) * 6.2831853
    cos, sin = torch.cos(ang), torch.sin(ang)
    kq = b.Quantizer(d=hd, dhat=32, depth=depth, K=K, grouping=b.STRIDED)
    vq = b.Quantizer(d=hd, dhat=32, depth=depth, K=K, grouping=b.CONTIGUOUS)
    kq.set_codebooks(Ck)
    vq.set_codebooks(Cv)
    wsb = b.rvq_attn_workspace_bytes(N, Hq, Hkv)
    ws = torch.empty(wsb // 4, device="cuda")
    out = torch.empty((Hq, hd), device="cuda")
    a, z = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, reps=20):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        z.record()
        torch.cuda.synchronize()
        return a.elapsed_time(z) / reps

    scale = 1.0 / hd ** 0.5
    fused = timed(lambda: b.rvq_attn_decode(kq.ctx, vq.ctx, qv, Hq, Hkv, kc, ks, vc, vs, N, cos, sin, scale,
                                            out, ws, wsb))
    kp, vp = kq.pack(kc), vq.pack(vc)  # 11 bytes per (row, group): the paper's storage
    fused_packed = timed(lambda: b.rvq_attn_decode(kq.ctx, vq.ctx, qv, Hq, Hkv, kp, ks, vp, vs, N, cos, sin,
                                                   scale, out, ws, wsb, packed=1))
    kx = torch.empty((rows, hd), dtype=torch.float16, device="cuda")
    vx = torch.empty((rows, hd), dtype=torch.float16, device="cuda")
    cosr = cos.repeat_interleave(Hkv, 0).contiguous()
    sinr = sin.repeat_interleave(Hkv, 0).contiguous()
    unfused = timed(lambda: (b.rvq_decode_rope(kq.ctx, kc, ks, rows, depth, cosr, sinr, hd, kx, hd),
                             b.rvq_decode(vq.ctx, vc, vs, rows, depth, vx, hd)))
    kq.close()
    vq.close()
    hbm = rows * (2 * (4 * depth * 2) + 2 * 2) + N * (hd // 2) * 4 * 2  # codes + std, rotary tables
    gather = rows * 2 * 4 * depth * 128                                 # codeword rows from L2
    return dict(workload="one query position over 131072 tokens x 8 kv heads (32 query heads), codes in the cache",
                fused_ms=fused, token_heads_per_s=rows / (fused * 1e-3),
                hbm_GBs=hbm / (fused * 1e-3) / 1e9, l2_gather_GBs=gather / (fused * 1e-3) / 1e9,
                fp16_kv_equivalent_GBs=rows * 2 * hd * 2 / (fused * 1e-3) / 1e9,
                fused_from_packed_records_ms=fused_packed, decode_k_and_v_to_fp16_ms=unfused)


def run_workload4(args):
    """Workload 4 (codebook learning): 1,048,576 mixture vectors, depth 8, K = 2048, stage by stage,
    10 (assign, update) rounds per stage + the assignment that forms the residuals; time per pass
    split into the assignment (rvq_encode over one stage) and the update (rvq_ema_update: scatter,
    reduction of the partial histograms, blend, refresh of the stage's derived copies)."""
    import torch

    from paper_2410_15704_amd import synth, train

    M, depth, K, iters = 1048576, 8, 2048, 10
    dR = torch.from_numpy(synth.gaussian_mixture(M)).cuda()

    class Timers:
        def __init__(self):
            self.ev, self.open = {}, {}

        def start(self, name):
            e = torch.cuda.Event(enable_timing=True)
            e.record()
            self.open[name] = e

        def stop(self, name):
            e = torch.cuda.Event(enable_timing=True)
            e.record()
            self.ev.setdefault(name, []).append((self.open.pop(name), e))

        def mean_ms(self, name):
            return sum(x.elapsed_time(y) for x, y in self.ev[name]) / len(self.ev[name])

    train.ema_train_sequential(dR, depth, K, 1, 0.99, 1e-5, seed=synth.BASE_SEED + 4)  # warm-up
    tm = Timers()
    a, z = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    train.ema_train_sequential(dR, depth, K, iters, 0.99, 1e-5, seed=synth.BASE_SEED + 4, timers=tm)
    z.record()
    torch.cuda.synchronize()
    assign_ms, update_ms = tm.mean_ms("assign"), tm.mean_ms("update")
    return dict(workload="workload 4: 1,048,576 vectors of 32, depth 8, K=2048, 10 rounds per stage, "
                         "decay 0.99, eps 1e-5, stage by stage",
                passes=depth * iters, schedule_ms=a.elapsed_time(z), assign_ms_per_pass=assign_ms,
                update_ms_per_pass=update_ms,
                assign_Mvec_s=M / (assign_ms * 1e-3) / 1e6,
                assign_frac_of_mfma_peak=2.0 * 32 * K * M / (assign_ms * 1e-3) / 1e12 / PEAK_MFMA_16BIT_TFLOPS,
                update_GBs=M * 130 / (update_ms * 1e-3) / 1e9)


def run_cpu_baseline(args):
    """The fp64 oracle, as it stands, on a bounded sample of workload 2 (encode + decode)."""
    import numpy as np

    import oracle
    from paper_2410_15704_amd import synth

    rows = args.cpu_rows
    N, d, dhat, depth, K = (W2[k] for k in ("N", "d", "dhat", "depth", "K"))
    Xb, _ = synth.llama_key(N, d, rows=slice(0, max(rows, 2048)))
    Xw = synth.widen(Xb, "bf16")
    Z = oracle.scaled_groups(Xw[:2048], dhat, oracle.STRIDED)
    C = oracle.sample_init_codebooks(Z, depth, K, np.random.Generator(np.random.PCG64(2)))
    C = C.astype(np.float32).astype(np.float64)
    t0 = time.perf_counter()
    r = oracle.encode(Xw[:rows], C, dhat, oracle.STRIDED)
    t1 = time.perf_counter()
    oracle.decode(r["codes"], r["std"], C, d, oracle.STRIDED)
    t2 = time.perf_counter()
    V = rows * (d // dhat)
    return dict(value=V / (t2 - t0) / 1e6, unit="Mvec/s", cores=oracle.threads(), kind="oracle",
                sample="first %d of 32768 rows of workload 2 (%d group vectors): oracle encode "
                       "%.2f s + decode %.2f s" % (rows, V, t1 - t0, t2 - t1),
                encode_Mvec_s=V / (t1 - t0) / 1e6)


def run_profile(args):
    """A few launches of one kernel, for `rocprofv3 --kernel-trace --stats` / `--pmc` runs.
    `copy` is a plain 1 GiB device copy whose FETCH_SIZE / WRITE_SIZE readings calibrate the
    counters' units."""
    import numpy as np
    import torch

    from paper_2410_15704_amd import binding as b
    from paper_2410_15704_amd import synth, train

    if args.profile == "copy":
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        return
    if args.profile == "attn":
        print(run_attn_decode(args))
        return
    if args.profile == "append":
        print(run_append(args))
        return
    if args.profile == "decode":
        T, d, G, depth, K = 16 * 32768, 1024, 32, 8, 2048
        Cs = torch.from_numpy(synth.decode_codebooks(2)).cuda()
        std = torch.from_numpy(synth.decode_std_fp16(T)).cuda()
        out = torch.empty((T, d), dtype=torch.float16, device="cuda")
        for s_, grp in enumerate((b.STRIDED, b.CONTIGUOUS)):
            q = b.Quantizer(d=d, dhat=32, depth=depth, K=K, out_dtype=b.F16, std_dtype=b.F16, grouping=grp)
            q.set_codebooks(Cs[s_])
            codes = synth.uniform_codes_device(T, G, depth, K, "cuda", extra=100 + s_)
            for _ in range(10):
                b.rvq_decode(q.ctx, codes, std, T, depth, out, d)
            torch.cuda.synchronize()
            q.close()
        return
    N, d, dhat, depth, K = (W2[k] for k in ("N", "d", "dhat", "depth", "K"))
    Xb, _ = synth.llama_key(N, d)
    dX = torch.from_numpy(Xb.view(np.int16)).cuda().view(torch.bfloat16)
    Zhead = train.scaled_groups(dX[:2048], d=d, dhat=dhat, grouping=b.STRIDED, in_dtype=b.BF16)
    C = train.sample_init_codebooks(Zhead, depth, K, seed=synth.BASE_SEED + 2)
    q = b.Quantizer(d=d, dhat=dhat, depth=depth, K=K, grouping=b.STRIDED, in_dtype=b.BF16,
                    out_dtype=b.F16, std_dtype=b.F16, encode_path=args.encode_path)
    q.set_codebooks(C)
    codes = torch.empty((N, d // dhat, depth), dtype=torch.int16, device="cuda")
    std = torch.empty((N,), dtype=torch.float16, device="cuda")
    if args.profile == "encode":
        for _ in range(25):
            b.rvq_encode(q.ctx, dX, N, d, 0, depth, codes, std, None)
    else:
        Z = train.scaled_groups(dX, d=d, dhat=dhat, grouping=b.STRIDED, in_dtype=b.BF16)
        b.rvq_encode(q.ctx, dX, N, d, 0, depth, codes, std, None)
        cs = torch.ones(K, dtype=torch.float32, device="cuda")
        es = C[0].clone()
        for _ in range(5):
            b.rvq_ema_update(q.ctx, 0, Z, codes, depth, N * (d // dhat), 0.99, 1e-5, cs, es)
    torch.cuda.synchronize()
    print(b.rvq_get_counters(q.ctx))
    q.close()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (rows shard across GPUs without "
              "communication, the moving-average update needs one all-reduce per stage); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.profile:
        run_profile(args)
        return
    r = run_steps(args)
    line = {
        "metric": "RVQ encode+decode+EMA step throughput, dhat=32, depth 8, K=2048 "
                  "(encode Mvec/s with matrix-core fraction, decode GB/s with HBM fraction inside)",
        "value": r["vec_per_step"] / (r["ms_per_step"] * 1e-3) / 1e6,
        "unit": "Mvec/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "workload 2: Llama-3-8B-like key projection, N=32768 x 1024 ch "
                               "bf16, strided groups of 32, depth 8, K=2048; encode + decode + "
                               "one EMA update of codebook 0 per step",
                   "vectors_per_step": r["vec_per_step"], "encode_path": args.encode_path},
        "breakdown": r["breakdown"],
        "roofline": r["roofline"],
    }
    if not args.no_decode_stream:
        line["decode_stream"] = run_decode_stream(args)
    if not args.no_extra_workloads:
        line["workload5"] = run_workload5(args)
        line["workload4"] = run_workload4(args)
        line["attn_decode"] = run_attn_decode(args)
        line["append"] = run_append(args)
    line["cpu_baseline"] = None if args.no_cpu else run_cpu_baseline(args)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
