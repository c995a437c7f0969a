"""Codebook-learning drivers composed from the library's entry points (host loops only; all
arithmetic of the method runs in librvq's kernels; torch is used for device memory, seeded index
draws and row gathers).

Section 3 of the paper: each codebook is initialised from "the corresponding inputs" (the paper
runs k-means on the first batch; the synthetic workloads sample K distinct rows instead) and is
then updated by an exponential moving average with decay 0.99.
"""
from __future__ import annotations

import torch

from . import binding as b


def scaled_groups(X: torch.Tensor, *, d: int, dhat: int, grouping: int, in_dtype: int,
                  scale: int = 1) -> torch.Tensor:
    """The vectors Algorithm 1 receives, float32 [N*G][dhat]: obtained from rvq_encode itself as
    the residual that a single all-zero codeword leaves."""
    q = b.Quantizer(d=d, dhat=dhat, depth=1, K=1, grouping=grouping, in_dtype=in_dtype,
                    scale=scale, std_dtype=b.F32)
    q.set_codebooks(torch.zeros((1, 1, dhat), dtype=torch.float32, device=X.device))
    _, _, res = q.encode(X, want_residual=True)
    torch.cuda.synchronize()
    q.close()
    return res.view(-1, dhat)


def sample_init_codebooks(Z: torch.Tensor, depth: int, K: int, seed: int,
                          encode_path: int = b.PATH_AUTO) -> torch.Tensor:
    """Stage-by-stage sample initialisation: codebook s = K distinct seeded rows of the vectors
    entering stage s; they are then quantized with it (rvq_encode, one stage) and the residuals
    go on to stage s + 1.  Z float32 [V][dhat] on the device.  Returns C [depth][K][dhat]."""
    V, dhat = Z.shape
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    C = torch.zeros((depth, K, dhat), dtype=torch.float32, device=Z.device)
    q = b.Quantizer(d=dhat, dhat=dhat, depth=depth, K=K, scale=0, encode_path=encode_path)
    R = Z.contiguous()
    codes = torch.empty((V, 1, depth), dtype=torch.int16, device=Z.device)
    for s in range(depth):
        pick = torch.randperm(V, generator=gen)[:K].sort().values.to(Z.device)
        C[s] = R.index_select(0, pick)
        q.set_codebooks(C)
        _, _, res = q.encode(R, want_residual=True, stages=(s, s + 1), codes=codes)
        R = res.view(V, dhat)
    torch.cuda.synchronize()
    q.close()
    return C


def ema_train_sequential(R0: torch.Tensor, depth: int, K: int, iters: int, decay: float,
                         eps: float, seed: int, encode_path: int = b.PATH_AUTO, timers=None,
                         picks=None):
    """Stage-by-stage residual training: for each stage, sample-initialise its codebook from the
    vectors entering it, run `iters` rounds of (assign, moving-average update) with state
    N_k = 1, M_k = C_k at the start, then assign once more and pass the residuals on.
    R0 float32 [M][dhat]; `picks[s]` (K row indices) replaces the seeded draw of stage s.
    Returns the learnt codebooks [depth][K][dhat]."""
    M, dhat = R0.shape
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    q = b.Quantizer(d=dhat, dhat=dhat, depth=depth, K=K, scale=0, encode_path=encode_path)
    C = torch.zeros((depth, K, dhat), dtype=torch.float32, device=R0.device)
    codes = torch.empty((M, 1, depth), dtype=torch.int16, device=R0.device)
    R = R0.contiguous()
    for s in range(depth):
        if picks is not None:
            pick = torch.as_tensor(picks[s], dtype=torch.int64, device=R.device)
        else:
            pick = torch.randperm(M, generator=gen)[:K].sort().values.to(R.device)
        C[s] = R.index_select(0, pick)
        q.set_codebooks(C)
        cs = torch.ones(K, dtype=torch.float32, device=R.device)
        es = C[s].clone()
        for _ in range(iters):
            if timers:
                timers.start("assign")
            q.encode(R, stages=(s, s + 1), codes=codes)
            if timers:
                timers.stop("assign")
                timers.start("update")
            b.rvq_ema_update(q.ctx, s, R, codes.data_ptr() + 2 * s, depth, M, decay, eps, cs, es)
            if timers:
                timers.stop("update")
        _, _, res = q.encode(R, want_residual=True, stages=(s, s + 1), codes=codes)
        R = res.view(M, dhat)
        C = q.get_codebooks()
    torch.cuda.synchronize()
    q.close()
    return C


def kmeans_init_codebooks(Z: torch.Tensor, depth: int, K: int, iters: int, picks,
                          encode_path: int = b.PATH_AUTO) -> torch.Tensor:
    """The initialisation Section 3 describes, stage by stage: the codebook of stage s starts
    from rows `picks[s]` (K indices) of the vectors entering stage s and is refined by `iters`
    Lloyd steps on them; a Lloyd step is rvq_encode over that one stage (assignment) followed by
    rvq_ema_update with decay 0 and no smoothing (each codeword becomes the mean of its vectors;
    one that no vector chose becomes 0).  The vectors are then quantized with the result and
    their residuals enter stage s + 1.  Z float32 [V][dhat] on the device.
    Returns C [depth][K][dhat]."""
    V, dhat = Z.shape
    q = b.Quantizer(d=dhat, dhat=dhat, depth=depth, K=K, scale=0, encode_path=encode_path)
    C = torch.zeros((depth, K, dhat), dtype=torch.float32, device=Z.device)
    codes = torch.empty((V, 1, depth), dtype=torch.int16, device=Z.device)
    R = Z.contiguous()
    for s in range(depth):
        pick = torch.as_tensor(picks[s], dtype=torch.int64, device=Z.device)
        C[s] = R.index_select(0, pick)
        q.set_codebooks(C)
        for _ in range(iters):
            q.encode(R, stages=(s, s + 1), codes=codes)
            cs = torch.zeros(K, dtype=torch.float32, device=Z.device)
            es = torch.zeros((K, dhat), dtype=torch.float32, device=Z.device)
            b.rvq_ema_update(q.ctx, s, R, codes.data_ptr() + 2 * s, depth, V, 0.0, 0.0, cs, es)
        _, _, res = q.encode(R, want_residual=True, stages=(s, s + 1), codes=codes)
        R = res.view(V, dhat)
        C = q.get_codebooks()
    torch.cuda.synchronize()
    q.close()
    return C


def ema_train_online(R0: torch.Tensor, depth: int, K: int, iters: int, decay: float, eps: float,
                     picks, encode_path: int = b.PATH_AUTO, batches=None,
                     init: torch.Tensor | None = None) -> torch.Tensor:
    """All stages in every step, as in the paper's training (Section 3): the codebooks start from
    picked rows stage by stage (sample initialisation); then `iters` steps, each walking the
    stages: assign with the current codebook (rvq_encode over that stage), pass on the residual
    formed with that pre-update codebook, update the codebook (rvq_ema_update).  Moving-average
    state N_k = 1, M_k = C_k at the start.  R0 float32 [M][dhat].  With `batches` (a callable:
    step -> float32 [M_t][dhat] on the device) every step works on a fresh batch, as the paper's
    training does, and R0 only serves the initialisation; `init` [depth][K][dhat] replaces the
    sample initialisation (e.g. by kmeans_init_codebooks).  Returns C [depth][K][dhat]."""
    M, dhat = R0.shape
    dev = R0.device
    q = b.Quantizer(d=dhat, dhat=dhat, depth=depth, K=K, scale=0, encode_path=encode_path)
    C = torch.zeros((depth, K, dhat), dtype=torch.float32, device=dev)
    codes = torch.empty((M, 1, depth), dtype=torch.int16, device=dev)
    R = R0.contiguous()
    if init is not None:
        C = init.to(device=dev, dtype=torch.float32).contiguous().clone()
        q.set_codebooks(C)
    else:
        for s in range(depth):
            C[s] = R.index_select(0, torch.as_tensor(picks[s], dtype=torch.int64, device=dev))
            q.set_codebooks(C)
            _, _, res = q.encode(R, want_residual=True, stages=(s, s + 1), codes=codes)
            R = res.view(M, dhat)
    cs = [torch.ones(K, dtype=torch.float32, device=dev) for _ in range(depth)]
    es = [C[s].clone() for s in range(depth)]
    for t in range(iters):
        R = (R0 if batches is None else batches(t)).contiguous()
        Mt = R.shape[0]
        if codes.shape[0] != Mt:
            codes = torch.empty((Mt, 1, depth), dtype=torch.int16, device=dev)
        for s in range(depth):
            _, _, res = q.encode(R, want_residual=True, stages=(s, s + 1), codes=codes)
            b.rvq_ema_update(q.ctx, s, R, codes.data_ptr() + 2 * s, depth, Mt, decay, eps, cs[s], es[s])
            R = res.view(Mt, dhat)
    C = q.get_codebooks()
    torch.cuda.synchronize()
    q.close()
    return C
