"""The enqueue calls under HIP graph capture: encode (both entry points), pack, decode (LDS and
row kernels, int16 codes and packed records), decode with the rotary embedding, the moving-average
update and attention over codes are captured once and replayed several times, with the inputs
changed and the program's own eager work and synchronisations between the replays.  Every replay
must give, bit for bit, what the same calls give when issued eagerly on the same inputs: the calls
allocate nothing, synchronise nothing and record no memset node, so a captured sequence is exactly
its kernels."""
import numpy as np
import pytest

from paper_2410_15704_amd import synth

pytestmark = pytest.mark.gpu

D, DEPTH, K, G = 1024, 8, 2048, 32
N = 16384          # N * G = 2^19: the strided decode takes the LDS kernel
HD, HKV, REP, NA = 128, 2, 4, 3000


def _sequence(b, torch, q, qc, kq, vq, bufs):
    """The calls under test, on the current stream, from `bufs["x"]` into the other buffers."""
    x = bufs["x"]
    b.rvq_encode(q.ctx, x, N, D, 0, DEPTH, bufs["codes"], bufs["std"], bufs["res"])
    b.rvq_encode_static(qc.ctx, x, N, D, 0, DEPTH, bufs["codes_c"], bufs["std_c"])
    b.rvq_pack_codes(q.ctx, bufs["codes"], N, bufs["packed"])
    b.rvq_decode(q.ctx, bufs["codes"], bufs["std"], N, DEPTH, bufs["out"], D)             # LDS kernel
    b.rvq_decode(qc.ctx, bufs["codes_c"], bufs["std_c"], N, DEPTH, bufs["out_c"], D)      # row kernel
    b.rvq_decode_packed(q.ctx, bufs["packed"], bufs["std"], N, DEPTH, bufs["out_p"], D)
    b.rvq_decode_rope(q.ctx, bufs["codes"], bufs["std"], N, DEPTH, bufs["cos"], bufs["sin"], HD,
                      bufs["out_r"], D)
    b.rvq_ema_update(q.ctx, 0, bufs["res"].view(N * G, 32), bufs["codes"], DEPTH, N * G, 0.99, 1e-5,
                     bufs["ema_n"], bufs["ema_s"])
    # attention of one query position over the first NA * HKV rows of the codes, read as heads of
    # 128 channels (any codes in range will do: both sides of the comparison read the same ones)
    b.rvq_attn_decode(kq.ctx, vq.ctx, bufs["q"], HKV * REP, HKV, bufs["codes"], bufs["std"],
                      bufs["codes_c"], bufs["std_c"], NA, bufs["cos"], bufs["sin"], 0.09, bufs["att"],
                      bufs["ws"], bufs["ws"].numel() * 4)


OUTPUTS = ("codes", "std", "res", "codes_c", "std_c", "packed", "out", "out_c", "out_p", "out_r",
           "ema_n", "ema_s", "att")


def test_captured_calls_replay_like_eager_ones(gpu_device):
    import torch

    from paper_2410_15704_amd import binding as b

    rows = [synth.llama_key(N, D, index=i)[0] for i in (11, 12, 13)]
    xs = [torch.from_numpy(r.view(np.int16)).cuda().view(torch.bfloat16) for r in rows]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(3)
    C = (torch.randn((DEPTH, K, 32), device="cuda", generator=gen) *
         (0.7 ** torch.arange(DEPTH, device="cuda"))[:, None, None]).contiguous()
    mk = lambda grouping, d=D: b.Quantizer(d=d, dhat=32, depth=DEPTH, K=K, grouping=grouping,
                                           in_dtype=b.BF16, std_dtype=b.F16, out_dtype=b.F16)
    # the moving-average update rewrites its context's codebook, so each run starts from C again
    q, qc, kq, vq = mk(b.STRIDED), mk(b.CONTIGUOUS), mk(b.STRIDED, HD), mk(b.CONTIGUOUS, HD)
    for t in (q, qc, kq, vq):
        t.set_codebooks(C)
    ang = torch.arange(N, device="cuda").double()[:, None] * \
        (10000.0 ** (-2.0 * torch.arange(HD // 2, device="cuda").double() / HD))[None, :]

    def buffers():
        z = lambda shape, dt: torch.zeros(shape, dtype=dt, device="cuda")
        wsb = b.rvq_attn_workspace_bytes(NA, HKV * REP, HKV)
        return dict(x=torch.empty_like(xs[0]), codes=z((N, G, DEPTH), torch.int16), std=z(N, torch.float16),
                    res=z((N, G, 32), torch.float32), codes_c=z((N, G, DEPTH), torch.int16),
                    std_c=z(N, torch.float16), packed=z((N, G, b.rvq_packed_record_bytes(q.ctx)), torch.uint8),
                    out=z((N, D), torch.float16), out_c=z((N, D), torch.float16),
                    out_p=z((N, D), torch.float16), out_r=z((N, D), torch.float16),
                    ema_n=z((K,), torch.float32), ema_s=z((K, 32), torch.float32),
                    att=z((HKV * REP, HD), torch.float32), ws=z(wsb // 4, torch.float32),
                    cos=torch.cos(ang).float(), sin=torch.sin(ang).float(),
                    q=torch.randn((HKV * REP, HD), device="cuda", generator=gen))

    eager, graph = buffers(), buffers()
    graph["q"].copy_(eager["q"])

    def reset(bufs, x):
        bufs["x"].copy_(x)
        bufs["ema_n"].fill_(1.0)
        bufs["ema_s"].copy_(C[0])
        q.set_codebooks(C)

    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    reset(graph, xs[0])
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=side):
        _sequence(b, torch, q, qc, kq, vq, graph)
    torch.cuda.synchronize()

    for rep, x in enumerate((xs[0], xs[1], xs[2], xs[1])):
        reset(eager, x)
        _sequence(b, torch, q, qc, kq, vq, eager)
        torch.cuda.synchronize()
        # eager work of the program's own between the replays
        junk = torch.randn((512, 512), device="cuda", generator=gen)
        assert torch.isfinite((junk @ junk).sum()).item()
        reset(graph, x)
        for name in OUTPUTS:
            if name not in ("ema_n", "ema_s"):
                graph[name].zero_()
        g.replay()
        torch.cuda.synchronize()
        for name in OUTPUTS:
            assert torch.equal(graph[name].view(torch.uint8), eager[name].view(torch.uint8)), \
                "replay %d: %s differs from the eager call" % (rep, name)
        assert int(eager["codes"].max()) > 0 and float(eager["att"].abs().max()) > 0
    assert b.rvq_check_kernels(q.ctx) == 0 and b.rvq_check_kernels(qc.ctx) == 0
    del g
    for t in (q, qc, kq, vq):
        t.close()
