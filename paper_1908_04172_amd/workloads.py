"""Seeded synthetic inputs shaped like the paper's layers (CryptoNets' convolution and dense
layers, appendix "Network Architectures"; the (N, L) triples of the appendix "SEAL Performance
Test").  This module only produces INPUTS: modulus chains, MAC plans (which ciphertext meets which
plaintext), uniform residues and Gaussian weights.  It contains none of the method's arithmetic and
is the one module both the GPU tests and the CPU oracle's tests draw their data from.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 190804172


# ----------------------------------------------------------------------------- moduli

def _is_prime(n: int) -> bool:
    if n < 2:
        return False
    small = (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37)
    for p in small:
        if n % p == 0:
            return n == p
    d, r = n - 1, 0
    while d % 2 == 0:
        d //= 2
        r += 1
    for a in small:
        x = pow(a, d, n)
        if x in (1, n - 1):
            continue
        for _ in range(r - 1):
            x = x * x % n
            if x == n - 1:
                break
        else:
            return False
    return True


def ntt_primes(bits: int, N: int, count: int) -> List[int]:
    """The `count` largest primes below 2**bits with p = 1 (mod 2N), in descending order."""
    out: List[int] = []
    step = 2 * N
    p = ((1 << bits) - 1) // step * step + 1
    while p >= (1 << bits):
        p -= step
    while len(out) < count:
        if p <= step:
            raise ValueError("ran out of candidates")
        if _is_prime(p):
            out.append(p)
        p -= step
    return out


def modulus_chain(bit_sizes: List[int], N: int) -> List[int]:
    """One prime per requested bit size, in the order given (limb 0 first; the last limb is the
    one a rescale drops); repeated sizes take successive primes, so all limbs are distinct."""
    need = {}
    for b in bit_sizes:
        need[b] = need.get(b, 0) + 1
    pools = {b: ntt_primes(b, N, c) for b, c in need.items()}
    used = {b: 0 for b in need}
    chain = []
    for b in bit_sizes:
        chain.append(pools[b][used[b]])
        used[b] += 1
    return chain


# ----------------------------------------------------------------------------- MAC plans

@dataclass
class Plan:
    """out[o] = sum over t in [off[o], off[o+1]) of ct_in[term_ct[t]] * pt[term_pt[t]]."""
    n_in: int
    n_out: int
    n_pt: int
    off: np.ndarray
    term_ct: np.ndarray
    term_pt: np.ndarray

    @property
    def n_terms(self) -> int:
        return int(self.term_ct.size)

    def subset(self, outputs) -> "Plan":
        """The plan restricted to the listed outputs (indices into ct_in / pt unchanged)."""
        outputs = list(outputs)
        off = [0]
        tc, tp = [], []
        for o in outputs:
            a, b = int(self.off[o]), int(self.off[o + 1])
            tc.append(self.term_ct[a:b])
            tp.append(self.term_pt[a:b])
            off.append(off[-1] + (b - a))
        cat = lambda xs: np.concatenate(xs).astype(np.uint32) if xs else np.zeros(0, np.uint32)
        return Plan(self.n_in, len(outputs), self.n_pt, np.asarray(off, np.uint32), cat(tc), cat(tp))


def dense_plan(K: int, M: int) -> Plan:
    """Dense K -> M: output o sums ct k times weight w[k][o]; plaintext index k*M + o."""
    off = (np.arange(M + 1, dtype=np.uint64) * K).astype(np.uint32)
    term_ct = np.tile(np.arange(K, dtype=np.uint32), M)
    o = np.repeat(np.arange(M, dtype=np.uint32), K)
    term_pt = term_ct * np.uint32(M) + o
    return Plan(K, M, K * M, off, term_ct, term_pt.astype(np.uint32))


def conv_plan(H: int, W: int, C: int, KH: int, KW: int, OC: int, stride: int, padding: str) -> Plan:
    """2-D convolution over an H x W x C tensor of ciphertexts (index (h*W + w)*C + c), weights
    [kh][kw][c][oc] (plaintext index ((kh*KW + kw)*C + c)*OC + oc), outputs (oh*OW + ow)*OC + oc.
    'valid': no padding.  'same': TensorFlow-style, out = ceil(in/stride), extra padding at the end;
    taps that fall on padding contribute nothing and are left out of the plan."""
    if padding == "valid":
        OH, OW = (H - KH) // stride + 1, (W - KW) // stride + 1
        pt_, pl_ = 0, 0
    elif padding == "same":
        OH, OW = -(-H // stride), -(-W // stride)
        pad_h = max((OH - 1) * stride + KH - H, 0)
        pad_w = max((OW - 1) * stride + KW - W, 0)
        pt_, pl_ = pad_h // 2, pad_w // 2
    else:
        raise ValueError(padding)
    off = [0]
    term_ct: List[int] = []
    term_pt: List[int] = []
    for oh in range(OH):
        for ow in range(OW):
            taps = []
            for kh in range(KH):
                h = oh * stride + kh - pt_
                if h < 0 or h >= H:
                    continue
                for kw in range(KW):
                    w = ow * stride + kw - pl_
                    if w < 0 or w >= W:
                        continue
                    for c in range(C):
                        taps.append(((h * W + w) * C + c, (kh * KW + kw) * C + c))
            for oc in range(OC):
                for ct_idx, w_idx in taps:
                    term_ct.append(ct_idx)
                    term_pt.append(w_idx * OC + oc)
                off.append(len(term_ct))
    return Plan(H * W * C, OH * OW * OC, KH * KW * C * OC, np.asarray(off, np.uint32),
                np.asarray(term_ct, np.uint32), np.asarray(term_pt, np.uint32))


# ----------------------------------------------------------------------------- the five configs

@dataclass
class Config:
    index: int                    # 1-based, as the configs are numbered
    name: str
    log2N: int
    bit_sizes: List[int]
    layer: str                    # 'dense' | 'conv'
    geometry: tuple
    pt_kind: str                  # 'scalar' | 'poly'
    log2_scale: int
    sigma: float
    has_bias: bool
    _plan: Optional[Plan] = field(default=None, repr=False)
    _q: Optional[List[int]] = field(default=None, repr=False)

    @property
    def N(self) -> int:
        return 1 << self.log2N

    @property
    def L(self) -> int:
        return len(self.bit_sizes)

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    @property
    def q(self) -> List[int]:
        if self._q is None:
            self._q = modulus_chain(self.bit_sizes, self.N)
        return self._q

    @property
    def plan(self) -> Plan:
        if self._plan is None:
            self._plan = dense_plan(*self.geometry) if self.layer == "dense" else conv_plan(*self.geometry)
        return self._plan


def configs() -> List[Config]:
    return [
        Config(1, "cfg1 dense 64->16, N=2^12, L=2x30b", 12, [30, 30], "dense", (64, 16), "scalar", 24, 0.1, True),
        Config(2, "cfg2 conv 28x28x1 5x5x5 s2 valid, N=2^13, L=60b+3x40b", 13, [60, 40, 40, 40], "conv",
               (28, 28, 1, 5, 5, 5, 2, "valid"), "scalar", 40, 0.1, True),
        Config(3, "cfg3 dense 845->100, N=2^13, L=60b+3x40b", 13, [60, 40, 40, 40], "dense", (845, 100),
               "scalar", 40, 0.05, True),
        Config(4, "cfg4 conv 32x32x3 3x3x16 s2 same, N=2^14, L=2x60b+6x50b", 14, [60, 60] + [50] * 6, "conv",
               (32, 32, 3, 3, 3, 16, 2, "same"), "scalar", 50, 0.1, True),
        Config(5, "cfg5 dense 256->64 full-poly pt, N=2^14, L=2x60b+6x50b", 14, [60, 60] + [50] * 6, "dense",
               (256, 64), "poly", 50, 0.0, False),
    ]


def config(index: int) -> Config:
    return configs()[index - 1]


# ----------------------------------------------------------------------------- random data

def uniform_residues(outer: Tuple[int, ...], q: List[int], N: int, seed: int) -> np.ndarray:
    """uint64 [*outer][len(q)][N], limb i uniform in [0, q[i]) (NumPy default_rng(seed))."""
    rng = np.random.default_rng(seed)
    out = np.empty(tuple(outer) + (len(q), N), dtype=np.uint64)
    for i, qi in enumerate(q):
        out[..., i, :] = rng.integers(0, qi, size=tuple(outer) + (N,), dtype=np.uint64)
    return out


def uniform_residues_torch(outer: Tuple[int, ...], q: List[int], N: int, seed: int, device, chunk: int = 64):
    """The same distribution generated on `device` with torch (for tensors too large to build on
    the host quickly): int64 [*outer][len(q)][N] whose bit patterns are the uint64 residues.
    Deterministic for a given (seed, device type); values differ from uniform_residues()."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    n = int(np.prod(outer)) if len(outer) else 1
    out = torch.empty((n, len(q), N), dtype=torch.int64, device=device)
    for i, qi in enumerate(q):
        for a in range(0, n, chunk):
            b = min(n, a + chunk)
            out[a:b, i, :] = torch.randint(0, int(qi), (b - a, N), dtype=torch.int64, device=device,
                                           generator=gen)
    return out.view(*outer, len(q), N)


def normal_values(n: int, sigma: float, seed: int) -> np.ndarray:
    """fp64 N(0, sigma) weights / biases."""
    return np.random.default_rng(seed).normal(0.0, sigma, size=n)
