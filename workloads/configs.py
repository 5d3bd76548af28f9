"""Input generators for the five benchmark configurations and for random test instances.

Every generator is a pure function of its seed and size arguments and returns an
``Instance``: the matrix (dense column-major, CSR, or a shared dense matrix for a
batch of instances), the target(s) b, the ascending value set D, a starting point
x0 in D^n, and the configured iteration count.  The real data sets of the paper
(model weights, calibration text, tomography image sets, filter baselines) are not
available offline; these inputs only take their shapes, value distributions and
structure:

* LLM weight quantisation (paper section "LLM Quantization W/O Outlier Separation"):
  every output row is an independent DMMV sharing the calibration matrix X.
* Discrete tomography (paper section "Discrete Tomography", Appendix D.4):
  parallel-beam projection matrix, few grey levels, uniform noise.
* FIR filter design (paper section "FIR Design with Discrete Coefficients"):
  cosine matrix on a frequency grid, fixed-point coefficient set.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

CONFIG_NAMES = {
    1: "dense_toy_256x64_f64",
    2: "fir_4096x32_f64_10bit",
    3: "tomography_256x256_180x363_csr_f32",
    4: "llm_layer_2048x4096_R4096_int4_f32",
    5: "llm_mlp_4096x4096_R11008_int3_f32",
}


@dataclass
class Instance:
    name: str
    kind: str                      # "dense" | "csr" | "batched"
    dtype: np.dtype
    m: int
    n: int
    D: np.ndarray                  # ascending, dtype
    b: np.ndarray                  # [m], or [R][m] for a batch
    x0: np.ndarray                 # [n] values in D, or [R][n]
    iters: int
    A: Optional[np.ndarray] = None          # dense m x n, Fortran (column-major) order
    csr_rowptr: Optional[np.ndarray] = None  # int64 [m+1]
    csr_col: Optional[np.ndarray] = None     # int32 [nnz], ascending inside a row
    csr_val: Optional[np.ndarray] = None     # dtype [nnz]
    R: int = 1
    scale: Optional[np.ndarray] = None       # [R] per-instance scale (batched), dtype
    meta: dict = field(default_factory=dict)

    @property
    def nd(self) -> int:
        return int(self.D.shape[0])

    @property
    def nnz(self) -> int:
        return int(self.csr_val.shape[0]) if self.csr_val is not None else self.m * self.n

    def moves_per_iter(self) -> int:
        """Non-null candidate moves scored per iteration (all instances)."""
        return self.R * self.n * (self.nd - 1)


# --------------------------------------------------------------------------------------
# helpers (input construction only)
# --------------------------------------------------------------------------------------
def _round_to_set(v: np.ndarray, D: np.ndarray) -> np.ndarray:
    """Nearest element of the ascending set D for every entry of v (ties -> lower)."""
    idx = np.searchsorted(D, v)
    idx = np.clip(idx, 1, len(D) - 1)
    lo = D[idx - 1]
    hi = D[idx]
    pick_hi = (hi - v) < (v - lo)
    return np.where(pick_hi, hi, lo)


def _chebyshev_lp(A: np.ndarray, b: np.ndarray, lo: float, hi: float):
    """Continuous relaxation min t s.t. -t <= Ax-b <= t, lo <= x <= hi (HiGHS)."""
    from scipy.optimize import linprog

    m, n = A.shape
    c = np.zeros(n + 1)
    c[-1] = 1.0
    A_ub = np.block([[A, -np.ones((m, 1))], [-A, -np.ones((m, 1))]])
    b_ub = np.concatenate([b, -b])
    bounds = [(lo, hi)] * n + [(0, None)]
    res = linprog(c, A_ub=A_ub, b_ub=b_ub, bounds=bounds, method="highs")
    if res.status != 0:
        return None, None
    return res.x[:n], float(res.x[-1])


# --------------------------------------------------------------------------------------
# config 1: dense toy
# --------------------------------------------------------------------------------------
def dense_toy(seed: int = 1001, m: int = 256, n: int = 64, iters: int = 200,
              dtype=np.float64) -> Instance:
    rng = np.random.default_rng(seed)
    D = np.arange(-8, 8, dtype=np.float64)
    A = rng.standard_normal((m, n))
    xs = rng.choice(D, size=n)
    b = A @ xs + rng.uniform(-0.5, 0.5, size=m)
    xls = np.linalg.lstsq(A, b, rcond=None)[0]
    x0 = np.clip(np.rint(xls), D[0], D[-1])
    return Instance(
        name=CONFIG_NAMES[1] if (m, n) == (256, 64) else f"dense_toy_{m}x{n}",
        kind="dense", dtype=np.dtype(dtype), m=m, n=n, D=D.astype(dtype),
        A=np.asfortranarray(A.astype(dtype)), b=b.astype(dtype), x0=x0.astype(dtype),
        iters=iters, meta={"seed": seed})


# --------------------------------------------------------------------------------------
# config 2: FIR low-pass, 32 free coefficients, 10-bit signed integers
# --------------------------------------------------------------------------------------
def fir_lowpass(seed: int = 1002, m: int = 4096, n: int = 32, bits: int = 10,
                iters: int = 500, dtype=np.float64) -> Instance:
    # frequency grid on [0, 0.2 pi] u [0.25 pi, pi], rows split in proportion to band widths
    m_pass = int(round(m * 0.2 / 0.95))
    m_stop = m - m_pass
    w = np.concatenate([np.linspace(0.0, 0.2 * np.pi, m_pass),
                        np.linspace(0.25 * np.pi, np.pi, m_stop)])
    j = np.arange(n, dtype=np.float64)
    A = 2.0 * np.cos(np.outer(w, j))
    half = 2 ** (bits - 1)
    b = np.concatenate([np.full(m_pass, float(half)), np.zeros(m_stop)])
    D = np.arange(-half, half, dtype=np.float64)
    xlp, tlp = _chebyshev_lp(A, b, D[0], D[-1])
    if xlp is None:
        xlp = np.linalg.lstsq(A, b, rcond=None)[0]
    x0 = np.clip(np.rint(xlp), D[0], D[-1])
    return Instance(
        name=CONFIG_NAMES[2] if (m, n, bits) == (4096, 32, 10) else f"fir_{m}x{n}_{bits}bit",
        kind="dense", dtype=np.dtype(dtype), m=m, n=n, D=D.astype(dtype),
        A=np.asfortranarray(A.astype(dtype)), b=b.astype(dtype), x0=x0.astype(dtype),
        iters=iters, meta={"seed": seed, "lp_bound": tlp, "m_pass": m_pass})


# --------------------------------------------------------------------------------------
# config 3: discrete tomography, parallel beam, CSR fp32
# --------------------------------------------------------------------------------------
def _phantom(rng: np.random.Generator, size: int, n_ellipses: int = 8) -> np.ndarray:
    img = np.zeros((size, size), dtype=np.float64)
    c = (size - 1) / 2.0
    yy, xx = np.mgrid[0:size, 0:size].astype(np.float64)
    s = size / 256.0
    for e in range(n_ellipses):
        rad = rng.uniform(0, 0.55) * (size / 2.0)
        ang = rng.uniform(0, 2 * np.pi)
        cx, cy = c + rad * np.cos(ang), c + rad * np.sin(ang)
        ax, ay = rng.uniform(10, 45, size=2) * s
        th = rng.uniform(0, np.pi)
        u = (xx - cx) * np.cos(th) + (yy - cy) * np.sin(th)
        v = -(xx - cx) * np.sin(th) + (yy - cy) * np.cos(th)
        img[(u / ax) ** 2 + (v / ay) ** 2 <= 1.0] = 0.5 if e % 2 == 0 else 1.0
    return img


def _parallel_beam_csr(size: int, n_angles: int, n_bins: int):
    """Exact line-length weights of unit-spaced rays through unit pixels.

    Row i = angle * n_bins + bin, column j = row-major pixel.  For direction
    (cos t, sin t) the chord of a ray at signed distance d from a pixel centre is a
    trapezoid in d: flat top 1/max(|c|,|s|) for |d| <= ||c|-|s||/2, falling linearly
    to 0 at |d| = (|c|+|s|)/2.
    """
    import scipy.sparse as sp

    c0 = (size - 1) / 2.0
    py, px = np.mgrid[0:size, 0:size]
    px = (px.ravel() - c0).astype(np.float64)
    py = (py.ravel() - c0).astype(np.float64)
    pix = np.arange(size * size, dtype=np.int64)
    centre_bin = (n_bins - 1) // 2
    rows, cols, vals = [], [], []
    for a in range(n_angles):
        t = a * np.pi / n_angles
        ct, st = np.cos(t), np.sin(t)
        ac, as_ = abs(ct), abs(st)
        w1 = 0.5 * (ac + as_)
        w2 = 0.5 * abs(ac - as_)
        top = 1.0 / max(ac, as_)
        p = px * ct + py * st                      # signed offset of the pixel centre
        base = np.floor(p).astype(np.int64)
        for off in (-1, 0, 1, 2):
            sb = base + off                        # ray offset (integer spaced)
            d = np.abs(sb - p)
            if w1 - w2 > 1e-15:
                ln = np.where(d <= w2, top, np.where(d < w1, top * (w1 - d) / (w1 - w2), 0.0))
            else:
                ln = np.where(d < w1, top, 0.0)
            b_idx = sb + centre_bin
            ok = (ln > 0.0) & (b_idx >= 0) & (b_idx < n_bins)
            rows.append(a * n_bins + b_idx[ok])
            cols.append(pix[ok])
            vals.append(ln[ok])
    rows = np.concatenate(rows)
    cols = np.concatenate(cols)
    vals = np.concatenate(vals)
    M = sp.csr_matrix((vals, (rows, cols)), shape=(n_angles * n_bins, size * size))
    M.sum_duplicates()
    M.sort_indices()
    return M


def tomography(seed: int = 1003, size: int = 256, n_angles: int = 180,
               n_bins: Optional[int] = None, iters: int = 2000, noise: float = 0.02,
               sirt_sweeps: int = 20, dtype=np.float32) -> Instance:
    rng = np.random.default_rng(seed)
    if n_bins is None:
        n_bins = 2 * int(np.ceil((size - 1) / 2.0 * np.sqrt(2.0))) + 1   # 363 for size 256
    D = np.array([0.0, 0.5, 1.0])
    xs = _phantom(rng, size).ravel()
    M = _parallel_beam_csr(size, n_angles, n_bins)
    Mt = M.astype(dtype).astype(np.float64)        # the matrix as stored (cast to dtype)
    clean = Mt @ xs
    b = clean + rng.uniform(-noise, noise, size=M.shape[0]) * clean.max()
    # starting point: a few SIRT sweeps from zero, rounded to the grey levels
    rs = np.asarray(Mt.sum(axis=1)).ravel()
    cs = np.asarray(Mt.sum(axis=0)).ravel()
    rinv = np.where(rs > 0, 1.0 / np.maximum(rs, 1e-30), 0.0)
    cinv = np.where(cs > 0, 1.0 / np.maximum(cs, 1e-30), 0.0)
    x = np.zeros(M.shape[1])
    MtT = Mt.T.tocsr()
    for _ in range(sirt_sweeps):
        x = x + cinv * (MtT @ (rinv * (b - Mt @ x)))
    x0 = _round_to_set(x, D)
    full = (size, n_angles) == (256, 180)
    return Instance(
        name=CONFIG_NAMES[3] if full else f"tomography_{size}x{size}_{n_angles}x{n_bins}",
        kind="csr", dtype=np.dtype(dtype), m=M.shape[0], n=M.shape[1], D=D.astype(dtype),
        csr_rowptr=M.indptr.astype(np.int64), csr_col=M.indices.astype(np.int32),
        csr_val=M.data.astype(dtype), b=b.astype(dtype), x0=x0.astype(dtype), iters=iters,
        meta={"seed": seed, "size": size, "n_angles": n_angles, "n_bins": n_bins,
              "phantom": xs.astype(dtype)})


# --------------------------------------------------------------------------------------
# configs 4 and 5: one linear layer, every output row an independent instance
# --------------------------------------------------------------------------------------
def _bf16_round(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even), returned as fp32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def llm_layer(seed: int, tokens: int, features: int, rows: int, bits: int, iters: int,
              bf16_activations: bool = False, name: Optional[str] = None,
              dtype=np.float32) -> Instance:
    rng = np.random.default_rng(seed)
    X = rng.standard_t(4.0, size=(tokens, features))
    n_out = max(1, int(round(0.01 * features)))
    hot = rng.choice(features, size=n_out, replace=False)
    X[:, hot] *= 20.0
    X = X.astype(np.float32)
    if bf16_activations:
        X = _bf16_round(X)
    W = (rng.standard_normal((rows, features)) * 0.02).astype(np.float32)
    half = 2 ** (bits - 1)
    D = np.arange(-half, half, dtype=np.float64)
    qmax = float(half - 1)
    scale = (np.abs(W).max(axis=1).astype(np.float64) / qmax).astype(np.float32)
    scale = np.maximum(scale, np.float32(1e-30))
    # targets b_r = X w_r accumulated in fp64, stored in the working precision
    B = (W.astype(np.float64) @ X.astype(np.float64).T)            # [rows][tokens]
    q0 = np.clip(np.rint(W.astype(np.float64) / scale.astype(np.float64)[:, None]),
                 D[0], D[-1])
    return Instance(
        name=name or f"llm_{tokens}x{features}_R{rows}_int{bits}",
        kind="batched", dtype=np.dtype(dtype), m=tokens, n=features, D=D.astype(dtype),
        A=np.asfortranarray(X.astype(dtype)), b=np.ascontiguousarray(B.astype(dtype)),
        x0=np.ascontiguousarray(q0.astype(dtype)), iters=iters, R=rows,
        scale=scale.astype(dtype),
        meta={"seed": seed, "bits": bits, "outlier_channels": np.sort(hot)})


# --------------------------------------------------------------------------------------
# random instances for unit / parity tests
# --------------------------------------------------------------------------------------
def random_dense(seed: int, m: int, n: int, nd: int, dtype=np.float64, integer: bool = False,
                 iters: int = 50) -> Instance:
    """Random dense instance.  integer=True gives small-integer data, for which every
    floating-point operation of the method is exact and exact score ties are frequent."""
    rng = np.random.default_rng(seed)
    if integer:
        A = rng.integers(-3, 4, size=(m, n)).astype(np.float64)
        D = np.sort(rng.choice(np.arange(-6, 7), size=nd, replace=False)).astype(np.float64)
        b = rng.integers(-20, 21, size=m).astype(np.float64)
    else:
        A = rng.standard_normal((m, n))
        D = np.sort(rng.uniform(-2, 2, size=nd))
        while np.any(np.diff(D.astype(dtype)) <= 0):
            D = np.sort(rng.uniform(-2, 2, size=nd))
        b = rng.standard_normal(m) * 3.0
    x0 = rng.choice(D, size=n) if n else np.zeros(0)
    return Instance(name=f"random_dense_{m}x{n}_nd{nd}_s{seed}", kind="dense",
                    dtype=np.dtype(dtype), m=m, n=n, D=D.astype(dtype),
                    A=np.asfortranarray(A.astype(dtype)), b=b.astype(dtype),
                    x0=x0.astype(dtype), iters=iters, meta={"seed": seed})


def random_sparse(seed: int, m: int, n: int, nd: int, density: float = 0.1,
                  dtype=np.float32, integer: bool = False, iters: int = 50,
                  explicit_zeros: bool = False) -> Instance:
    import scipy.sparse as sp

    rng = np.random.default_rng(seed)
    mask = rng.uniform(size=(m, n)) < density
    if integer:
        V = rng.integers(-3, 4, size=(m, n)).astype(np.float64)
        if not explicit_zeros:
            V[V == 0] = 1.0
        D = np.sort(rng.choice(np.arange(-6, 7), size=nd, replace=False)).astype(np.float64)
        b = rng.integers(-20, 21, size=m).astype(np.float64)
    else:
        V = rng.standard_normal((m, n))
        D = np.sort(rng.uniform(-2, 2, size=nd))
        while np.any(np.diff(D.astype(dtype)) <= 0):
            D = np.sort(rng.uniform(-2, 2, size=nd))
        b = rng.standard_normal(m) * 3.0
    rows, cols = np.nonzero(mask)
    vals = V[rows, cols]
    order = np.lexsort((cols, rows))
    rows, cols, vals = rows[order], cols[order], vals[order]
    rowptr = np.zeros(m + 1, dtype=np.int64)
    np.add.at(rowptr, rows + 1, 1)
    rowptr = np.cumsum(rowptr)
    x0 = rng.choice(D, size=n) if n else np.zeros(0)
    return Instance(name=f"random_sparse_{m}x{n}_nd{nd}_s{seed}", kind="csr",
                    dtype=np.dtype(dtype), m=m, n=n, D=D.astype(dtype),
                    csr_rowptr=rowptr, csr_col=cols.astype(np.int32),
                    csr_val=vals.astype(dtype), b=b.astype(dtype), x0=x0.astype(dtype),
                    iters=iters, meta={"seed": seed})


def random_batched(seed: int, m: int, n: int, R: int, nd: int, dtype=np.float32,
                   integer: bool = False, iters: int = 30) -> Instance:
    rng = np.random.default_rng(seed)
    if integer:
        X = rng.integers(-3, 4, size=(m, n)).astype(np.float64)
        D = np.sort(rng.choice(np.arange(-6, 7), size=nd, replace=False)).astype(np.float64)
        B = rng.integers(-20, 21, size=(R, m)).astype(np.float64)
        scale = rng.choice(np.array([0.5, 1.0, 2.0]), size=R)
    else:
        X = rng.standard_t(4.0, size=(m, n))
        D = (np.arange(nd) - nd // 2).astype(np.float64)
        scale = rng.uniform(0.005, 0.02, size=R)
        B = (rng.standard_normal((R, n)) * 0.02) @ X.T
    x0 = rng.choice(D, size=(R, n))
    return Instance(name=f"random_batched_{m}x{n}_R{R}_nd{nd}_s{seed}", kind="batched",
                    dtype=np.dtype(dtype), m=m, n=n, D=D.astype(dtype),
                    A=np.asfortranarray(X.astype(dtype)),
                    b=np.ascontiguousarray(B.astype(dtype)),
                    x0=np.ascontiguousarray(x0.astype(dtype)), iters=iters, R=R,
                    scale=scale.astype(dtype), meta={"seed": seed})


# --------------------------------------------------------------------------------------
def make_config(idx: int, size: str = "full") -> Instance:
    """Benchmark configuration idx in 1..5.  size="small" keeps the structure and the
    value distributions but shrinks the dimensions so the CPU oracle finishes in seconds."""
    small = size == "small"
    if idx == 1:
        return dense_toy(1001)
    if idx == 2:
        return fir_lowpass(1002, m=520, n=12, bits=6, iters=80) if small else fir_lowpass(1002)
    if idx == 3:
        if small:
            return tomography(1003, size=40, n_angles=24, iters=120)
        return tomography(1003)
    if idx == 4:
        if small:
            return llm_layer(1004, tokens=200, features=96, rows=70, bits=4, iters=25)
        return llm_layer(1004, tokens=2048, features=4096, rows=4096, bits=4, iters=100,
                         name=CONFIG_NAMES[4])
    if idx == 5:
        if small:
            return llm_layer(1005, tokens=136, features=80, rows=45, bits=3, iters=25,
                             bf16_activations=True)
        return llm_layer(1005, tokens=4096, features=4096, rows=11008, bits=3, iters=300,
                         bf16_activations=True, name=CONFIG_NAMES[5])
    raise ValueError(f"config index {idx} not in 1..5")
