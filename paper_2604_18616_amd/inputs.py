"""Seeded synthetic inputs for the attention-forward workloads.

This module holds no attention arithmetic: it only produces the Q/K/V bit
patterns (and sampled query-row lists) that both the HIP path and the CPU
reference are fed, so that the two always see identical bits.

Recipe: a splitmix64 counter stream -> two 32-bit uniforms per draw ->
Box-Muller normal in fp64 -> scale by sigma (+ optional shift) -> fp32 -> bf16
round-to-nearest-even.  Draw order per workload: Q, K, V, then the per-head key
shift if the workload has one.  Values and shapes mirror the paper's attention
workload (Evaluation, "Kernel Performance": bf16, causal GQA prefill shapes, synthetic data).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

_M64 = (1 << 64) - 1


def splitmix64(counter: np.ndarray, seed: int) -> np.ndarray:
    """splitmix64 output for state = seed + (counter+1)*golden-gamma (vectorised, uint64)."""
    with np.errstate(over="ignore"):
        z = (counter.astype(np.uint64) + np.uint64(1)) * np.uint64(0x9E3779B97F4A7C15) + np.uint64(seed & _M64)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def normal_stream(seed: int, start: int, n: int) -> np.ndarray:
    """n iid N(0,1) draws (fp64) at stream positions start .. start+n-1."""
    out = np.empty(n, dtype=np.float64)
    chunk = 1 << 22
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        r = splitmix64(np.arange(start + lo, start + hi, dtype=np.uint64), seed)
        u1 = ((r >> np.uint64(32)).astype(np.float64) + 1.0) * (1.0 / 4294967296.0)   # (0, 1]
        u2 = (r & np.uint64(0xFFFFFFFF)).astype(np.float64) * (1.0 / 4294967296.0)    # [0, 1)
        out[lo:hi] = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return out


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even.  Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    u = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> fp32 (exact)."""
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    Sq: int
    Sk: int
    D: int
    causal: bool
    seed: int
    sigma: float = 1.0
    k_shift: bool = False          # add one N(0,1) constant per kv head to K before rounding
    check_rows: int = 0            # 0 = every row is cheap enough to check; else rows per head

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.D))

    def flops(self) -> float:
        """Algorithmic FLOPs: 4*D per visible (query, key) pair."""
        if not self.causal:
            pairs = self.Sq * self.Sk
        else:
            i = np.arange(self.Sq, dtype=np.int64)
            pairs = int(np.clip(i + (self.Sk - self.Sq) + 1, 0, self.Sk).sum())
        return 4.0 * self.D * self.B * self.Hq * pairs

    def dense_flops(self) -> float:
        """The paper's 'effective' convention (Evaluation, "Ablation Study"): dense FLOPs incl. masked pairs."""
        return 4.0 * self.D * self.B * self.Hq * self.Sq * self.Sk

    def bytes(self) -> float:
        """Compulsory HBM bytes: Q, O (bf16), K, V (bf16), LSE (fp32)."""
        return (2 * self.B * self.Hq * self.Sq * self.D * 2 + 2 * self.B * self.Hkv * self.Sk * self.D * 2
                + 4 * self.B * self.Hq * self.Sq)


# The five benchmark configurations, in the order the baseline file lists them.
WORKLOADS = {
    "C1": Workload("C1", 1, 2, 2, 128, 128, 64, False, 1001),
    "C2": Workload("C2", 16, 16, 16, 1024, 1024, 128, False, 1002),
    "C3": Workload("C3", 4, 32, 8, 4096, 4096, 128, True, 1003),
    "C4": Workload("C4", 2, 16, 16, 8192, 8192, 64, False, 1004, sigma=0.5, k_shift=True, check_rows=512),
    "C5": Workload("C5", 1, 32, 8, 32768, 32768, 128, True, 1005, check_rows=256),
}


# Further shapes: the paper's own attention workload (Evaluation, "Kernel Performance"; Figure 3a: causal GQA, batch 16, 8 query
# heads on 1 kv head, d = 128, sequence 1024 .. 16384) and a long non-causal case that
# isolates the steady state of the kernels (no diagonal, no ragged last wave of workgroups).
for _s in (1024, 2048, 4096, 8192, 16384):
    WORKLOADS["P%d" % _s] = Workload("P%d" % _s, 16, 8, 1, _s, _s, 128, True, 2000 + _s, check_rows=64)
WORKLOADS["N8K"] = Workload("N8K", 1, 32, 8, 8192, 8192, 128, False, 3001, check_rows=64)


def make_qkv(w: Workload):
    """Q [B,Hq,Sq,D], K, V [B,Hkv,Sk,D] as uint16 arrays of bf16 bit patterns."""
    nq = w.B * w.Hq * w.Sq * w.D
    nk = w.B * w.Hkv * w.Sk * w.D
    q = (normal_stream(w.seed, 0, nq) * w.sigma).astype(np.float32)
    k = (normal_stream(w.seed, nq, nk) * w.sigma).astype(np.float32)
    v = (normal_stream(w.seed, nq + nk, nk) * w.sigma).astype(np.float32)
    k = k.reshape(w.B, w.Hkv, w.Sk, w.D)
    if w.k_shift:
        c = normal_stream(w.seed, nq + 2 * nk, w.Hkv).astype(np.float32)
        k = k + c.reshape(1, w.Hkv, 1, 1)
    return (f32_to_bf16_bits(q).reshape(w.B, w.Hq, w.Sq, w.D),
            f32_to_bf16_bits(k).reshape(w.B, w.Hkv, w.Sk, w.D),
            f32_to_bf16_bits(v).reshape(w.B, w.Hkv, w.Sk, w.D))


def sample_rows(w: Workload, n: int) -> np.ndarray:
    """Query rows to check per (b, h): int32 [B*Hq, n], sorted.

    Always contains the tile-edge / causal-extreme rows {0,1,63,64,127,128,255,256,
    Sq-2,Sq-1} that exist; the rest is drawn without replacement from a splitmix64
    stream seeded with seed ^ (b*Hq + h).
    """
    n = min(n, w.Sq)
    forced = sorted({r for r in (0, 1, 63, 64, 127, 128, 255, 256, w.Sq - 2, w.Sq - 1) if 0 <= r < w.Sq})[:n]
    out = np.empty((w.B * w.Hq, n), dtype=np.int32)
    for bh in range(w.B * w.Hq):
        keys = splitmix64(np.arange(w.Sq, dtype=np.uint64), (w.seed ^ bh) + 0x5EED)
        keys[np.asarray(forced, dtype=np.int64)] = 0          # forced rows sort first
        order = np.argsort(keys, kind="stable")
        out[bh] = np.sort(order[:n])
    return out


# ---------------------------------------------------------------------------------------
# GEMM workloads (the paper's Evaluation, "Kernel Performance": square bf16 matrices with normally distributed
# entries).  Same generator; draw order A, then B.  b_is_nk: B is stored [N,K] (a linear
# layer's weight, C = A W^T) instead of [K,N].
# ---------------------------------------------------------------------------------------
@dataclass(frozen=True)
class GemmWorkload:
    name: str
    M: int
    N: int
    K: int
    seed: int
    b_is_nk: bool = False
    sigma: float = 1.0

    def flops(self) -> float:
        return 2.0 * self.M * self.N * self.K

    def bytes(self) -> float:
        """Compulsory HBM bytes: A, B read once, C written once (all bf16)."""
        return 2.0 * (self.M * self.K + self.K * self.N + self.M * self.N)


GEMM_WORKLOADS = {}
for _s in (1024, 2048, 4096, 8192, 16384):
    GEMM_WORKLOADS["G%d" % _s] = GemmWorkload("G%d" % _s, _s, _s, _s, 4000 + _s)
    GEMM_WORKLOADS["G%dT" % _s] = GemmWorkload("G%dT" % _s, _s, _s, _s, 4000 + _s, b_is_nk=True)


def make_ab(w: GemmWorkload):
    """A [M,K] and B ([K,N], or [N,K] if w.b_is_nk) as uint16 arrays of bf16 bit patterns."""
    na, nb = w.M * w.K, w.K * w.N
    a = f32_to_bf16_bits((normal_stream(w.seed, 0, na) * w.sigma).astype(np.float32)).reshape(w.M, w.K)
    b = f32_to_bf16_bits((normal_stream(w.seed, na, nb) * w.sigma).astype(np.float32))
    return a, b.reshape((w.N, w.K) if w.b_is_nk else (w.K, w.N))


def sample_outputs(w: GemmWorkload, n: int):
    """n output coordinates (i, j) to check: tile corners and edges that exist, then seeded draws."""
    edge_i = sorted({x for x in (0, 1, 31, 32, 127, 128, 255, 256, w.M - 2, w.M - 1) if 0 <= x < w.M})
    edge_j = sorted({x for x in (0, 1, 31, 32, 63, 64, 255, 256, w.N - 2, w.N - 1) if 0 <= x < w.N})
    forced = [(i, j) for i in edge_i for j in edge_j][:n]
    r = splitmix64(np.arange(max(0, n - len(forced)), dtype=np.uint64), w.seed + 0x5EED)
    si = np.array([p[0] for p in forced] + list((r >> np.uint64(32)) % np.uint64(w.M)), dtype=np.int32)
    sj = np.array([p[1] for p in forced] + list((r & np.uint64(0xFFFFFFFF)) % np.uint64(w.N)), dtype=np.int32)
    return si, sj


# ---------------------------------------------------------------------------------------
# Fused-MoE workloads (the paper's Evaluation, "Kernel Performance": block-quantized FP8 feed-forward experts, model
# dimension 7168, intermediate dimension 2048, top-4 routing, 32 experts per GPU under 8-way
# expert parallelism).  The paper gives the shape only; the rest is this build's recipe:
#   x        [T,H] bf16, iid N(0,1);
#   routing  each token draws 4 distinct experts out of E*EP global ones; the ids handed to the
#            library are local (0..E-1) or -1 for experts that live on another GPU; the 4
#            weights are positive and sum to 1;
#   weights  e4m3 codes whose values are round(64 * N(0,1)) in e4m3 (16-bit inverse-CDF draws),
#            block scales (one per 128 x 128 block) = (1 + u/4) / (64 sqrt(fan_in)), u in [0,1).
# The encoder below serves input generation only (nearest value, table search).
# ---------------------------------------------------------------------------------------
def e4m3_values() -> np.ndarray:
    """The 256 e4m3 code values as fp64 (NaN for the two NaN codes)."""
    c = np.arange(256)
    e, m = (c >> 3) & 15, (c & 7).astype(np.float64)
    v = np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * 2.0 ** (e.astype(np.float64) - 7))
    v = np.where((e == 15) & ((c & 7) == 7), np.nan, v)
    return np.where(c >= 128, -v, v)


def nearest_e4m3(v: np.ndarray) -> np.ndarray:
    """Nearest e4m3 code of each value (|v| clamped to 448); for building inputs only."""
    pos = e4m3_values()[:127]                      # 0 .. 448, ascending
    a = np.minimum(np.abs(v), 448.0)
    hi = np.clip(np.searchsorted(pos, a), 1, 126)
    lo = hi - 1
    code = np.where(a - pos[lo] <= pos[hi] - a, lo, hi).astype(np.uint8)
    return np.where(v < 0, code | 0x80, code).astype(np.uint8)


_CODE_TABLE = None


def _normal_code_table() -> np.ndarray:
    global _CODE_TABLE
    if _CODE_TABLE is None:
        from statistics import NormalDist
        nd = NormalDist()
        z = np.array([nd.inv_cdf((u + 0.5) / 65536.0) for u in range(65536)])
        _CODE_TABLE = nearest_e4m3(64.0 * z)
    return _CODE_TABLE


def random_e4m3(seed: int, n: int) -> np.ndarray:
    """n e4m3 codes with values ~ 64 * N(0,1), four per splitmix64 draw."""
    table = _normal_code_table()
    out = np.empty((n + 3) // 4 * 4, dtype=np.uint8)
    chunk = 1 << 22
    for lo in range(0, out.size // 4, chunk):
        hi = min(out.size // 4, lo + chunk)
        r = splitmix64(np.arange(lo, hi, dtype=np.uint64), seed)
        for q in range(4):
            out[4 * lo + q:4 * hi:4] = table[((r >> np.uint64(16 * q)) & np.uint64(0xFFFF)).astype(np.int64)]
    return out[:n]


@dataclass(frozen=True)
class MoeWorkload:
    name: str
    T: int
    seed: int
    H: int = 7168
    I: int = 2048
    E: int = 32          # experts on this GPU
    KTOP: int = 4
    EP: int = 8          # expert-parallel ranks: E * EP experts in total

    def local_slots(self, ids: np.ndarray) -> int:
        return int((ids >= 0).sum())

    def flops(self, ids: np.ndarray) -> float:
        """Algorithmic FLOPs: 2 * (2I*H + H*I) per routed (token, local expert) pair."""
        return 6.0 * self.H * self.I * self.local_slots(ids)

    def bytes(self, ids: np.ndarray) -> float:
        """Compulsory HBM bytes: x read and y written (bf16), the weights of the experts that
        receive a token read once (1 byte each), routing tables."""
        used = len(set(ids[ids >= 0].tolist()))
        return 4.0 * self.T * self.H + 3.0 * self.H * self.I * used + 8.0 * self.T * self.KTOP


MOE_WORKLOADS = {("M%d" % _t): MoeWorkload("M%d" % _t, _t, 5000 + _t) for _t in (1024, 2048, 4096, 8192, 16384)}


def make_moe(w: MoeWorkload):
    """dict with x [T,H] (bf16 bits), ids [T,KTOP] int32, wts [T,KTOP] fp32, w13 [E,2I,H] and
    w2 [E,H,I] (e4m3 codes), s13 [E,2I/128,H/128] and s2 [E,H/128,I/128] (fp32)."""
    T, H, I, E, K = w.T, w.H, w.I, w.E, w.KTOP
    x = f32_to_bf16_bits(normal_stream(w.seed, 0, T * H).astype(np.float32)).reshape(T, H)
    total = E * w.EP
    keys = splitmix64(np.arange(T * total, dtype=np.uint64), w.seed + 1).reshape(T, total)
    glob = np.argsort(keys, axis=1, kind="stable")[:, :K]                  # K distinct experts per token
    ids = np.where(glob < E, glob, -1).astype(np.int32)                    # rank 0 owns experts 0..E-1
    u = (splitmix64(np.arange(T * K, dtype=np.uint64), w.seed + 2) >> np.uint64(40)).astype(np.float64) / 2.0 ** 24 + 0.25
    wts = (u.reshape(T, K) / u.reshape(T, K).sum(axis=1, keepdims=True)).astype(np.float32)
    w13 = random_e4m3(w.seed + 3, E * 2 * I * H).reshape(E, 2 * I, H)
    w2 = random_e4m3(w.seed + 4, E * H * I).reshape(E, H, I)

    def scales(seed, shape, fan_in):
        n = int(np.prod(shape))
        uu = (splitmix64(np.arange(n, dtype=np.uint64), seed) >> np.uint64(40)).astype(np.float64) / 2.0 ** 24
        return ((1.0 + uu / 4.0) / (64.0 * np.sqrt(fan_in))).astype(np.float32).reshape(shape)

    s13 = scales(w.seed + 5, (E, 2 * I // 128, H // 128), H)
    s2 = scales(w.seed + 6, (E, H // 128, I // 128), I)
    return dict(x=x, ids=ids, wts=wts, w13=w13, s13=s13, w2=w2, s2=s2)


def sample_tokens(w: MoeWorkload, ids: np.ndarray, n: int) -> np.ndarray:
    """n tokens to check: the first and last token, then seeded draws weighted toward tokens that
    have at least one local expert (the others must come out as exact zeros and cost nothing)."""
    order = np.argsort(splitmix64(np.arange(w.T, dtype=np.uint64), w.seed + 7), kind="stable")
    local = order[(ids[order] >= 0).any(axis=1)]
    remote = order[~(ids[order] >= 0).any(axis=1)]
    pick = [0, w.T - 1] + local[:max(0, n - 2 - min(4, len(remote)))].tolist() + remote[:4].tolist()
    return np.array(sorted(set(pick))[:n], dtype=np.int32)
