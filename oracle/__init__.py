"""fp64 CPU oracle for the RVQ KV-cache compressor (arXiv 2410.15704).

TEST INFRASTRUCTURE ONLY: imported by tests/, by ``__graft_entry__.smoke`` and
by the ``cpu_baseline`` leg of ``bench.py``.  The product package never imports
this module and this module never imports the product package.

The arithmetic lives in ``rvq_oracle.c`` (plain C, double precision, compiled
with gcc); this file only marshals numpy arrays into it.  Function names and
argument order mirror the C file; see its header for the paper passages each
function follows and for the readings taken where the paper is silent.  Two functions are
written out here in numpy on top of the C routines: ``decode_rope`` (the rotation of decoded pairs)
and ``attn_decode`` (softmax attention of one query over decoded keys and values).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import sys

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rvq_oracle.c")
_LIB = os.path.join(_HERE, "liborvq.so")

CONTIGUOUS = 0
STRIDED = 1


def build(force: bool = False) -> str:
    """Compile rvq_oracle.c with gcc into oracle/liborvq.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c_dp = ctypes.POINTER(ctypes.c_double)
        c_ip = ctypes.POINTER(ctypes.c_int32)
        i64, i32, f64 = ctypes.c_int64, ctypes.c_int, ctypes.c_double
        lib.rvq_oracle_threads.restype = i32
        lib.rvq_oracle_row_std.argtypes = [c_dp, i64, i64, i32, c_dp]
        lib.rvq_oracle_encode.argtypes = [c_dp, i64, i64, i64, i32, i64, i32, i32, i32, c_dp, c_ip,
                                          c_dp, c_dp, c_dp, c_dp]
        lib.rvq_oracle_decode.argtypes = [c_ip, c_dp, i64, i64, i64, i32, i32, i64, i32, c_dp, c_dp]
        lib.rvq_oracle_prefix_excess.argtypes = [c_dp, i64, i64, i64, i32, i64, i32, i32, i32, c_dp,
                                                 c_ip, c_dp, c_dp]
        lib.rvq_oracle_ema_update.argtypes = [c_dp, c_ip, i64, i64, i64, i64, f64, f64, c_dp, c_dp,
                                              c_dp]
        lib.rvq_oracle_compressed_bits.argtypes = [i64, i64, i32, i64, i32]
        lib.rvq_oracle_compressed_bits.restype = i64
        _lib = lib
    return _lib


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if a is not None else None


def _ip(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)) if a is not None else None


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def threads() -> int:
    """Number of OpenMP threads the row loops use."""
    return int(_load().rvq_oracle_threads())


def row_std(X, ddof: int = 0):
    X = _f64(X)
    N, d = X.shape
    out = np.empty(N, dtype=np.float64)
    _check(_load().rvq_oracle_row_std(_dp(X), N, d, ddof, _dp(out)), "row_std")
    return out


def encode(X, C, dhat: int, grouping: int = CONTIGUOUS, scale: bool = True, ddof: int = 0,
           want_residual: bool = False, want_gap: bool = False):
    """Section 2.2 + Algorithm 1.  X [N][d]; C [depth][K][dhat].

    Returns a dict: codes int32 [N][G][depth], std [N], and when asked
    residual [N][G][dhat], gap and rnorm2 [N][G][depth].
    """
    X = _f64(X)
    C = _f64(C)
    N, d = X.shape
    depth, K, dh = C.shape
    if dh != dhat:
        raise ValueError("codebook width differs from dhat")
    G = d // dhat
    codes = np.empty((N, G, depth), dtype=np.int32)
    std = np.empty(N, dtype=np.float64)
    resid = np.empty((N, G, dhat), dtype=np.float64) if want_residual else None
    gap = np.empty((N, G, depth), dtype=np.float64) if want_gap else None
    rn2 = np.empty((N, G, depth), dtype=np.float64) if want_gap else None
    _check(_load().rvq_oracle_encode(_dp(X), N, d, dhat, depth, K, grouping, int(bool(scale)), ddof,
                                     _dp(C), _ip(codes), _dp(std), _dp(resid), _dp(gap), _dp(rn2)),
           "encode")
    out = {"codes": codes, "std": std}
    if want_residual:
        out["residual"] = resid
    if want_gap:
        out["gap"] = gap
        out["rnorm2"] = rn2
    return out


def decode(codes, std, C, d: int, grouping: int = CONTIGUOUS, depth_used: int | None = None):
    """Section 2.2, last sentence.  codes [N][G][depth]; std [N]; returns [N][d] float64."""
    codes = np.ascontiguousarray(codes, dtype=np.int32)
    std = _f64(std)
    C = _f64(C)
    depth, K, dhat = C.shape
    N = codes.shape[0]
    if codes.shape != (N, d // dhat, depth):
        raise ValueError("codes shape does not match [N][d/dhat][depth]")
    if depth_used is None:
        depth_used = depth
    out = np.empty((N, d), dtype=np.float64)
    _check(_load().rvq_oracle_decode(_ip(codes), _dp(std), N, d, dhat, depth, depth_used, K,
                                     grouping, _dp(C), _dp(out)), "decode")
    return out


def prefix_excess(X, C, dhat: int, given_codes, grouping: int = CONTIGUOUS, scale: bool = True,
                  ddof: int = 0):
    """dist(given code) - min dist per (vector, group, stage), residual rebuilt from the given
    codes of earlier stages; also the squared norm of that residual."""
    X = _f64(X)
    C = _f64(C)
    N, d = X.shape
    depth, K, _ = C.shape
    given = np.ascontiguousarray(given_codes, dtype=np.int32)
    G = d // dhat
    if given.shape != (N, G, depth):
        raise ValueError("given codes shape does not match [N][G][depth]")
    excess = np.empty((N, G, depth), dtype=np.float64)
    rn2 = np.empty((N, G, depth), dtype=np.float64)
    _check(_load().rvq_oracle_prefix_excess(_dp(X), N, d, dhat, depth, K, grouping,
                                            int(bool(scale)), ddof, _dp(C), _ip(given),
                                            _dp(excess), _dp(rn2)), "prefix_excess")
    return excess, rn2


def ema_update(R, codes, K: int, decay: float, eps: float, cluster_size, embed_sum):
    """One moving-average update of one codebook.  Returns new (cluster_size, embed_sum, codebook);
    the inputs are not modified."""
    R = _f64(R)
    M, dhat = R.shape
    codes = np.ascontiguousarray(codes, dtype=np.int32).reshape(-1)
    if codes.shape[0] != M:
        raise ValueError("one code per vector expected")
    cs = _f64(cluster_size).copy()
    es = _f64(embed_sum).copy()
    cb = np.empty((K, dhat), dtype=np.float64)
    _check(_load().rvq_oracle_ema_update(_dp(R), _ip(codes), 1, M, K, dhat, float(decay),
                                         float(eps), _dp(cs), _dp(es), _dp(cb)), "ema_update")
    return cs, es, cb


def compressed_bits(d: int, dhat: int, depth: int, K: int, std_bits: int = 16) -> int:
    return int(_load().rvq_oracle_compressed_bits(d, dhat, depth, K, std_bits))


def scaled_groups(X, dhat: int, grouping: int = CONTIGUOUS, scale: bool = True, ddof: int = 0):
    """The vectors Algorithm 1 receives: rows scaled by their std and split into groups,
    [N*G][dhat] float64.  Obtained from the C oracle itself, as the residual a single all-zero
    codeword leaves."""
    zero = np.zeros((1, 1, dhat), dtype=np.float64)
    out = encode(X, zero, dhat, grouping, scale=scale, ddof=ddof, want_residual=True)
    return out["residual"].reshape(-1, dhat)


def sample_init_codebooks(Z, depth: int, K: int, rng: np.random.Generator):
    """Stage-by-stage codebooks for the synthetic workloads: stage s takes K distinct rows, drawn
    without replacement, of the vectors that enter stage s (the scaled group vectors for s = 0,
    then the residuals the earlier stages leave).  Z [V][dhat] float64, V >= K.
    Returns C [depth][K][dhat] float64.  (Section 3 initialises each codebook from "the
    corresponding inputs"; sampling stands in for the k-means the paper runs on them.)"""
    Z = _f64(Z)
    V, dhat = Z.shape
    C = np.empty((depth, K, dhat), dtype=np.float64)
    R = Z
    for s in range(depth):
        pick = rng.choice(V, size=K, replace=False)
        C[s] = R[np.sort(pick)]
        out = encode(R, C[s:s + 1], dhat, CONTIGUOUS, scale=False, want_residual=True)
        R = out["residual"].reshape(V, dhat)
    return C


def kmeans_init_codebooks(Z, depth: int, K: int, iters: int, picks):
    """Section 3's initialisation, stage by stage: the codebook of stage s starts from K rows
    `picks[s]` of the vectors entering stage s and is refined by `iters` Lloyd steps on those
    vectors (assign every vector to its nearest codeword, replace each codeword by the mean of
    its vectors); the vectors are then quantized with the result and their residuals enter stage
    s + 1.  A Lloyd step is the moving-average update with decay 0 and no smoothing, so a
    codeword that no vector chose becomes 0 (no revival).  Z [V][dhat] float64.
    Returns (C [depth][K][dhat] float64, mse [depth][iters + 1]): mean squared quantization
    error of each stage before the first step and after every step."""
    Z = _f64(Z)
    V, dhat = Z.shape
    C = np.empty((depth, K, dhat), dtype=np.float64)
    mse = np.empty((depth, iters + 1), dtype=np.float64)
    R = Z
    for s in range(depth):
        Cs = R[np.asarray(picks[s])].copy()
        for it in range(iters):
            out = encode(R, Cs[None], dhat, CONTIGUOUS, scale=False, want_residual=True)
            mse[s, it] = np.mean(out["residual"] ** 2)
            _, _, Cs = ema_update(R, out["codes"].reshape(V), K, 0.0, 0.0,
                                  np.zeros(K), np.zeros((K, dhat)))
        out = encode(R, Cs[None], dhat, CONTIGUOUS, scale=False, want_residual=True)
        mse[s, iters] = np.mean(out["residual"] ** 2)
        C[s] = Cs
        R = out["residual"].reshape(V, dhat)
    return C, mse


def ema_train(R0, depth: int, K: int, iters: int, decay: float, eps: float, picks,
              schedule: str = "sequential", batches=None, progress=None):
    """Codebook learning by exponential moving average (Sections 2.1 and 3: decay 0.99) on a fixed
    set of vectors R0 [M][dhat], with moving-average state N_k = 1, M_k = C_k at the start.
      "sequential": stage by stage: codebook s starts from rows picks[s] of the vectors entering
          stage s, then `iters` rounds of (assign, update); a last assignment leaves the residuals
          that enter stage s + 1.
      "online" (all stages in every step, as in the paper's training): codebooks start from picked
          rows stage by stage (sample initialisation); then `iters` steps, each walking the stages:
          assign with the current codebook, pass on the residual formed with that (pre-update)
          codebook, update the codebook.  With `batches` (a list of `iters` arrays [M_t][dhat])
          step t works on batches[t] instead of R0, as the paper's training does with a fresh
          batch of tokens in every step; R0 then only serves the initialisation.
    `progress`, if given, is called with a short text after every stage ("sequential") or step
    ("online"); it sees no data and changes nothing.
    Returns C [depth][K][dhat] float64."""
    R0 = _f64(R0)
    M, dhat = R0.shape
    C = np.zeros((depth, K, dhat), dtype=np.float64)

    def assign(R, Cs):
        out = encode(R, Cs[None], dhat, CONTIGUOUS, scale=False, want_residual=True)
        return out["codes"].reshape(R.shape[0]), out["residual"].reshape(R.shape[0], dhat)

    if schedule == "sequential":
        R = R0
        for s in range(depth):
            Cs = R[np.asarray(picks[s])].copy()
            cs, es = np.ones(K), Cs.copy()
            for _ in range(iters):
                codes, _ = assign(R, Cs)
                cs, es, Cs = ema_update(R, codes, K, decay, eps, cs, es)
            _, R = assign(R, Cs)
            C[s] = Cs
            if progress:
                progress(f"oracle: stage {s} trained")
        return C
    if schedule != "online":
        raise ValueError(schedule)
    R = R0
    for s in range(depth):
        C[s] = R[np.asarray(picks[s])]
        _, R = assign(R, C[s])
    cs = [np.ones(K) for _ in range(depth)]
    es = [C[s].copy() for s in range(depth)]
    for t in range(iters):
        R = R0 if batches is None else _f64(batches[t])
        for s in range(depth):
            codes, Rn = assign(R, C[s])
            cs[s], es[s], C[s] = ema_update(R, codes, K, decay, eps, cs[s], es[s])
            R = Rn
        if progress:
            progress(f"oracle: step {t} done")
    return C


def rope_tables(positions, head_dim: int, base: float = 10000.0):
    """cos / sin of the rotary position embedding the paper cites (RoFormer): pair i of a head is
    turned by the angle position * base**(-2 i / head_dim).  Returns (cos, sin) float64
    [len(positions)][head_dim // 2].  Only used to build inputs; both sides receive the tables."""
    pos = np.asarray(positions, dtype=np.float64)[:, None]
    inv = base ** (-2.0 * np.arange(head_dim // 2, dtype=np.float64) / head_dim)[None, :]
    ang = pos * inv
    return np.cos(ang), np.sin(ang)


def decode_rope(codes, std, C, d: int, grouping: int, cos, sin, head_dim: int,
                depth_used: int | None = None):
    """Decode followed by the rotary position embedding (the paper quantizes keys BEFORE the
    rotary embedding, Section 3, so every decoded key is rotated before use): within every head
    of head_dim channels, the pair (x[2i], x[2i+1]) becomes
    (x[2i] cos_i - x[2i+1] sin_i, x[2i] sin_i + x[2i+1] cos_i), cos / sin float [N][head_dim/2]."""
    x = decode(codes, std, C, d, grouping, depth_used)
    N = x.shape[0]
    cos = _f64(cos)
    sin = _f64(sin)
    heads = d // head_dim
    xr = x.reshape(N, heads, head_dim // 2, 2)
    out = np.empty_like(xr)
    c = cos[:, None, :]
    s_ = sin[:, None, :]
    out[..., 0] = xr[..., 0] * c - xr[..., 1] * s_
    out[..., 1] = xr[..., 0] * s_ + xr[..., 1] * c
    return out.reshape(N, d)


def attn_decode(q, kcodes, kstd, Ck, k_grouping: int, vcodes, vstd, Cv, v_grouping: int,
                cos, sin, scale: float, n_kv_heads: int):
    """Attention of one query position over a cache that holds RVQ codes instead of keys and
    values (Section 3: one quantizer for the key and one for the value projection of an attention
    block, applied before the rotary embedding; the Conclusion names the cost of decoding inside
    attention as the open efficiency question).  Head vectors of hd = q.shape[1] channels are the
    rows of both quantizers: row n * n_kv_heads + h is head h of token n.

      k[n,h] = rotate(decode(kcodes, kstd)[n * Hkv + h], cos[n], sin[n])    (decode_rope)
      v[n,h] = decode(vcodes, vstd)[n * Hkv + h]
      s[a,n] = scale * q[a] . k[n, a // rep]          rep = Hq // Hkv query heads per kv head
      p[a,:] = softmax over n of s[a,:]
      out[a] = sum_n p[a,n] v[n, a // rep]

    Plain definition in float64, no blocking, the softmax with its maximum subtracted.
    q [Hq][hd]; codes [N * Hkv][hd / 32][depth]; std [N * Hkv]; cos, sin [N][hd / 2].
    Returns [Hq][hd] float64."""
    q = _f64(q)
    Hq, hd = q.shape
    Hkv = int(n_kv_heads)
    if Hq % Hkv:
        raise ValueError("query heads must be a multiple of kv heads")
    rep = Hq // Hkv
    rows = np.asarray(kcodes).shape[0]
    if rows % Hkv or np.asarray(vcodes).shape[0] != rows:
        raise ValueError("rows must be tokens x kv heads for both caches")
    N = rows // Hkv
    if N < 1:
        raise ValueError("attention over an empty cache is undefined")
    cos = _f64(cos)
    sin = _f64(sin)
    # every head of a token is turned by that token's angles
    k = decode_rope(kcodes, kstd, Ck, hd, k_grouping, np.repeat(cos, Hkv, axis=0),
                    np.repeat(sin, Hkv, axis=0), hd).reshape(N, Hkv, hd)
    v = decode(vcodes, vstd, Cv, hd, v_grouping).reshape(N, Hkv, hd)
    out = np.empty((Hq, hd), dtype=np.float64)
    for a in range(Hq):
        h = a // rep
        s = float(scale) * (k[:, h, :] @ q[a])
        w = np.exp(s - s.max())
        out[a] = (w / w.sum()) @ v[:, h, :]
    return out


def code_bits(K: int) -> int:
    """Bits of one stored code: the smallest b >= 1 with 2**b >= K (Section 3.2 counts log2 K)."""
    b = 1
    while (1 << b) < K:
        b += 1
    return b


def pack_codes(codes, K: int):
    """Packed code storage: the depth codes of one (token, group) written one after the other,
    b = code_bits(K) bits each, least significant bit first, into ceil(depth * b / 8) bytes
    (unused high bits of the last byte are 0).  codes int [N][G][depth] -> uint8 [N][G][bytes].
    Written as a bit matrix so that it can be checked by eye."""
    codes = np.asarray(codes).astype(np.int64)
    N, G, depth = codes.shape
    b = code_bits(K)
    rec = (depth * b + 7) // 8
    bit = np.zeros((N, G, rec * 8), dtype=np.uint8)
    for i in range(depth):
        for t in range(b):
            bit[:, :, i * b + t] = (codes[:, :, i] >> t) & 1
    return np.packbits(bit, axis=2, bitorder="little")


def unpack_codes(packed, K: int, depth: int):
    """Inverse of pack_codes: uint8 [N][G][bytes] -> int32 [N][G][depth]."""
    packed = np.asarray(packed, dtype=np.uint8)
    b = code_bits(K)
    bit = np.unpackbits(packed, axis=2, bitorder="little").astype(np.int64)
    codes = np.zeros(packed.shape[:2] + (depth,), dtype=np.int64)
    for i in range(depth):
        for t in range(b):
            codes[:, :, i] |= bit[:, :, i * b + t] << t
    return codes.astype(np.int32)


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
