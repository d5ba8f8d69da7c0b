"""Seeded synthetic inputs shared by the HIP path's tests/bench and by the CPU oracle.

This module only draws random inputs (numpy, host memory). It holds none of the
method's arithmetic and imports neither the HIP binding nor the oracle.

The workloads stand in for the LLM fine-tuning gradients of the paper's experiments
(Sec. 5; LLaMA/Mistral attention and MLP matrices), which need datasets and trained
weights: chunk counts and lengths follow the weight shapes, values are heavy-tailed
(Student-t) with per-row / per-layer scale spread to mimic outlier rows.
"""
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    cfg: int          # index used in the seed
    C: int            # chunks
    d: int            # chunk length
    r: int            # measurements per chunk (length of each compressed moment)
    k: int            # non-zeros kept / recovered per chunk
    grad: str         # "f32" | "bf16"
    matrix: str       # "stored" | "philox"
    steps: int
    dist: str         # "normal" | "student"
    nu: float = 3.0
    scale: float = 1.0
    a_seed: int = 1

    @property
    def n(self):
        return self.C * self.d


# the five configurations of the benchmark definition
CFG1 = Workload("cfg1_single_chunk", 1, 1, 4096, 256, 32, "f32", "stored", 1, "normal")
CFG2 = Workload("cfg2_64x65536", 2, 64, 65536, 2048, 256, "f32", "stored", 10, "student", 3.0, 1e-3)
CFG3 = Workload("cfg3_attn_4096x4096", 3, 1024, 16384, 1024, 64, "f32", "philox", 1, "student_rowscale")
CFG4 = Workload("cfg4_llama7b_block", 4, 12352, 16384, 1024, 64, "f32", "philox", 1, "student_layerscale")
CFG5 = Workload("cfg5_stress_bf16", 5, 128, 262144, 8192, 1024, "bf16", "philox", 1, "student", 2.5)
# not part of the benchmark definition: the paper's own memory-efficient setting (App. D: 256 chunks per
# 4096 x 4096 weight, one non-zero per chunk, kappa = 8) on the same Llama-2-7B block as configuration 4
CFG6 = Workload("paper_mesgc_llama7b_block", 6, 3088, 65536, 8, 1, "f32", "philox", 1, "student_layerscale")
CONFIGS = {1: CFG1, 2: CFG2, 3: CFG3, 4: CFG4, 5: CFG5, 6: CFG6}

# shapes of the linear weights of one Llama-2-7B block (rows, cols), cfg4
LLAMA7B_BLOCK = [(4096, 4096)] * 4 + [(4096, 11008)] * 2 + [(11008, 4096)]


def shrink(w, **kw):
    """A smaller workload with the same recipe (for cases the oracle must finish in seconds)."""
    return replace(w, **kw)


def _rng(*key):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(x) for x in key])))


def f32_to_bf16_bits(a):
    """Round-to-nearest-even conversion float32 -> bfloat16 bit patterns (uint16)."""
    b = np.ascontiguousarray(a, np.float32).view(np.uint32)
    rounded = b + (np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(h):
    return (np.ascontiguousarray(h, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def gradients(w, step=1, chunks=None):
    """Gradient chunks [C, d] for one step: float32, or uint16 bf16 bit patterns.

    `chunks` selects a subset of chunk indices (each chunk has its own seed, so a
    subset equals the corresponding rows of the full draw).
    """
    ids = range(w.C) if chunks is None else chunks
    out = np.empty((len(ids), w.d), np.float32)
    if w.dist == "student_layerscale":
        # chunks are laid out layer after layer; a shrunk workload keeps the proportions
        sizes = np.array([a * b for a, b in LLAMA7B_BLOCK], np.float64)
        bounds = np.cumsum(sizes) / sizes.sum()
        lay = _rng(w.cfg, 0, 7)
        layer_scale = np.exp(lay.uniform(np.log(1e-4), np.log(1e-2), size=len(sizes)))
    for o, c in enumerate(ids):
        g = _rng(w.cfg, step, c)
        if w.dist == "normal":
            x = g.standard_normal(w.d)
        else:
            x = g.standard_t(w.nu, w.d)
        if w.dist == "student_rowscale":
            # a 4096-wide matrix flattened row-major: d/4096 rows per chunk, one
            # log-normal(sigma=1) scale per row
            cols = 4096
            rows = max(1, w.d // cols)
            s = np.exp(g.standard_normal(rows))
            x = (x.reshape(rows, -1) * s[:, None]).reshape(-1)
        elif w.dist == "student_layerscale":
            layer = int(np.searchsorted(bounds, (c + 0.5) / w.C, side="left"))
            x = x * layer_scale[min(layer, len(sizes) - 1)]
        out[o] = (x * w.scale).astype(np.float32)
    if w.grad == "bf16":
        return f32_to_bf16_bits(out)
    return out


def ulp_cluster_gradients(seed, C, d, k):
    """Chunks [C, d] whose k-th largest magnitude sits inside a cluster of values one unit in the last place
    apart: about 3k entries with magnitudes 1.5 + j ulp (j in a window of about 2k/3 values, so every
    magnitude occurs several times: ties and one-ulp neighbours), random signs, plus about 2k/3 clearly
    larger entries and small noise elsewhere. An input generator for top-k tests, nothing more."""
    g = _rng(4242, seed, d, k)
    out = (g.standard_normal((C, d)) * 0.01).astype(np.float32)
    base = np.float32(1.5).view(np.uint32)
    for c in range(C):
        cluster = g.choice(d, size=min(d, 3 * k), replace=False)
        bits = base + g.integers(0, max(2, 2 * k // 3), size=cluster.size).astype(np.uint32)
        out[c, cluster] = bits.view(np.float32) * g.choice([-1.0, 1.0], size=cluster.size).astype(np.float32)
        rest = np.setdiff1d(np.arange(d), cluster)
        big = g.choice(rest, size=max(0, min(rest.size, k - k // 3)), replace=False)
        out[c, big] = (10.0 + g.random(big.size)).astype(np.float32)
    return out


def gaussian_matrix(seed, d, r):
    """At [d, r] float32 with iid N(0, 1/r) entries (the stored-matrix mode; Sec. 4.3)."""
    g = _rng(1000003, seed)
    a = g.standard_normal((d, r), dtype=np.float32)
    a *= np.float32(1.0 / np.sqrt(r))
    return a


def weights(w, chunks=None):
    """Initial weights W [C*d] float32 (small normal values)."""
    C = w.C if chunks is None else len(chunks)
    g = _rng(w.cfg, 424242)
    return (0.02 * g.standard_normal(C * w.d, dtype=np.float32)).astype(np.float32)


def sparse_signal(seed, d, k, lo=0.5, hi=2.0):
    """An exactly k-sparse vector in R^d with magnitudes in [lo, hi] and random signs."""
    g = _rng(77, seed)
    pos = np.sort(g.choice(d, size=k, replace=False)).astype(np.int32)
    mag = g.uniform(lo, hi, size=k) * g.choice([-1.0, 1.0], size=k)
    x = np.zeros(d, np.float64)
    x[pos] = mag
    return x, pos


def orthonormal_rows(seed, rho, m):
    """B [rho, m] float32 with orthonormal rows: the Q factor of a Gaussian matrix (an input of the
    CESGC tests; in the paper B holds leading singular vectors of a gradient, Sec. 4.4)."""
    g = _rng(555, seed)
    q, _ = np.linalg.qr(g.standard_normal((m, rho)))
    return np.ascontiguousarray(q.T.astype(np.float32))


def matrix_gradient(seed, step, m, n, basis, decay=0.7, noise=0.02):
    """Gradient of an m x n weight matrix for the CESGC workload: a fixed column space (`basis`,
    [R, m] with orthonormal rows, e.g. orthonormal_rows) with geometrically decaying strengths and
    heavy-tailed coefficients that change every step, plus dense Student-t noise. The first rows
    of `basis` are, by construction, the leading left singular directions a truncated SVD of the
    gradient would return, so they serve as the projection B without running an SVD here."""
    g = _rng(556, seed, step)
    R = basis.shape[0]
    strength = (decay ** np.arange(R)).astype(np.float32)
    coeff = g.standard_t(3.0, size=(R, n)).astype(np.float32) * strength[:, None]
    out = basis.T.astype(np.float32) @ coeff
    out += np.float32(noise) * g.standard_t(3.0, size=(m, n)).astype(np.float32)
    return np.ascontiguousarray(out * np.float32(1e-3))
