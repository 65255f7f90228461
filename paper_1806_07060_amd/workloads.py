"""Seeded synthetic workloads: GEMM cases and their host operands.

This module only *describes* and *draws* inputs; it holds none of the method's
arithmetic and imports neither the GPU library nor the oracle, so both sides of
a parity test can be fed from it.  The cases stand in for the paper's
workloads (rectangular DNN-like shapes and the synthetic (M, N, K) grids of
Section 4.1), which are not reproduced here.

Every case carries its own seed, derived from one base seed, the configuration
index and the case index; operands are drawn on the host with numpy's PCG64 in
fp32 so the CPU and the GPU see identical bits.
"""
from dataclasses import dataclass, replace
import math

import numpy as np

BASE_SEED = 180607060

ROW_MAJOR, COL_MAJOR = 101, 102
NO_TRANS, TRANS, CONJ_TRANS = 111, 112, 113

C_SENTINEL = np.float32(-7.25)  # value planted in the padding of C; must survive a call untouched


@dataclass(frozen=True)
class GemmCase:
    M: int
    N: int
    K: int
    transA: int = NO_TRANS
    transB: int = NO_TRANS
    alpha: float = 1.0
    beta: float = 0.0
    layout: int = COL_MAJOR
    lda: int = 0  # 0 = tight
    ldb: int = 0
    ldc: int = 0
    dist: str = "uniform"  # "uniform" = U[-1,1]; "normal_rsqrtk" = N(0, std 1/sqrt(K)); "smallint" = integers in [-8, 8]
    c0: str = "uniform"  # "uniform", "zero", "nan" (for beta == 0 checks), or same keys as dist
    seed: int = BASE_SEED
    name: str = ""

    # stored (rows, cols) of each operand
    def a_shape(self):
        return (self.K, self.M) if self.transA != NO_TRANS else (self.M, self.K)

    def b_shape(self):
        return (self.N, self.K) if self.transB != NO_TRANS else (self.K, self.N)

    def c_shape(self):
        return (self.M, self.N)

    def _min_ld(self, shape):
        return max(1, shape[0] if self.layout == COL_MAJOR else shape[1])

    def resolved(self):
        """Same case with tight leading dimensions filled in where they were 0."""
        return replace(self, lda=self.lda or self._min_ld(self.a_shape()), ldb=self.ldb or self._min_ld(self.b_shape()),
                       ldc=self.ldc or self._min_ld(self.c_shape()))

    def flops(self):
        return 2 * self.M * self.N * self.K

    def algorithmic_bytes(self):
        """Each operand once, C written once and read once iff beta != 0."""
        return 4 * (self.M * self.K + self.K * self.N + self.M * self.N * (2 if self.beta != 0.0 else 1))

    def tA(self):
        return int(self.transA != NO_TRANS)

    def tB(self):
        return int(self.transB != NO_TRANS)


def case_seed(config_index, case_index):
    """Per-case seed: a fixed mix of (base, config, case); stable across runs and platforms."""
    ss = np.random.SeedSequence([BASE_SEED, int(config_index), int(case_index)])
    return int(ss.generate_state(1, dtype=np.uint64)[0] >> np.uint64(1))


# ------------------------------------------------------------------------------------------
# operands
# ------------------------------------------------------------------------------------------

def buffer_len(layout, shape, ld):
    """Elements of the flat buffer that holds a rows x cols matrix with leading dimension ld."""
    rows, cols = shape
    outer = cols if layout == COL_MAJOR else rows
    return max(1, ld * outer)


def matrix_view(buf, layout, shape, ld):
    """rows x cols numpy view (logical indexing [r, c]) of a flat buffer; shares memory."""
    rows, cols = shape
    if layout == COL_MAJOR:
        return buf[: ld * cols].reshape(cols, ld).T[:rows, :] if cols else np.empty((rows, 0), buf.dtype)
    return buf[: ld * rows].reshape(rows, ld)[:, :cols] if rows else np.empty((0, cols), buf.dtype)


def _draw(rng, dist, shape, K):
    if dist == "uniform":
        return rng.uniform(-1.0, 1.0, size=shape).astype(np.float32)
    if dist == "normal_rsqrtk":
        return (rng.standard_normal(size=shape) / math.sqrt(max(K, 1))).astype(np.float32)
    if dist == "smallint":
        return rng.integers(-8, 9, size=shape).astype(np.float32)
    if dist == "zero":
        return np.zeros(shape, np.float32)
    if dist == "ones":
        return np.ones(shape, np.float32)
    if dist == "nan":
        return np.full(shape, np.nan, np.float32)
    raise ValueError(dist)


def make_operands(case, poison=True):
    """Flat fp32 host buffers (A, B, C0) for a case.

    The logical regions are drawn from the case's distribution; with `poison`
    the padding between the stored rows and the leading dimension holds NaN in
    A and B (reading it corrupts the result) and C_SENTINEL in C (writing it is
    detectable).
    """
    c = case.resolved()
    rng = np.random.Generator(np.random.PCG64(c.seed))
    out = []
    for shape, ld, dist, fill in ((c.a_shape(), c.lda, c.dist, np.nan), (c.b_shape(), c.ldb, c.dist, np.nan),
                                  (c.c_shape(), c.ldc, c.c0, C_SENTINEL)):
        buf = np.full(buffer_len(c.layout, shape, ld), fill if poison else 0.0, dtype=np.float32)
        v = matrix_view(buf, c.layout, shape, ld)
        if v.size:
            v[...] = _draw(rng, dist, shape, c.K)
        out.append(buf)
    return tuple(out)


def logical_max_abs(buf, layout, shape, ld):
    v = matrix_view(buf, layout, shape, ld)
    return float(np.max(np.abs(v))) if v.size else 0.0


# ------------------------------------------------------------------------------------------
# the five workload configurations
# ------------------------------------------------------------------------------------------

def config0():
    """One small square product: M = N = K = 64, no transposes, alpha 1, beta 0, C zero-initialised."""
    return [GemmCase(64, 64, 64, alpha=1.0, beta=0.0, dist="uniform", c0="zero", seed=case_seed(0, 0), name="cfg0/64")]


_T = {"N": NO_TRANS, "T": TRANS}


def config1(sizes=(256, 512, 1024, 2048, 4096, 8192)):
    """Square sweep, all four transpose combinations, alpha 1, beta 0.5, tight leading dimensions."""
    cases = []
    for n in sizes:
        for ta in "NT":
            for tb in "NT":
                cases.append(GemmCase(n, n, n, _T[ta], _T[tb], 1.0, 0.5, dist="uniform", c0="uniform",
                                      seed=case_seed(1, len(cases)), name=f"cfg1/{n}{ta}{tb}"))
    return cases


def config2():
    """Skinny products shaped like fully-connected layers at small batch; inputs N(0, std 1/sqrt(K))."""
    cases = []
    for M in (1024, 2048, 4096, 7680):
        for N in (1, 4, 16, 32, 64, 128):
            for K in (1024, 2048, 4096):
                for ta in "NT":
                    cases.append(GemmCase(M, N, K, _T[ta], NO_TRANS, 1.0, 0.0, dist="normal_rsqrtk", c0="zero",
                                          seed=case_seed(2, len(cases)), name=f"cfg2/{M}x{N}x{K}{ta}N"))
    return cases


def config3():
    """Convolution-lowered products: M = output channels, N = output pixels x batch, K = input channels x 9."""
    cases = []
    for M in (32, 64, 128, 256, 512):
        for N in (3136, 12544, 50176):
            for K in (27, 288, 576, 1152, 2304):
                cases.append(GemmCase(M, N, K, NO_TRANS, NO_TRANS, 1.0, 0.0, dist="uniform", c0="zero",
                                      seed=case_seed(3, len(cases)), name=f"cfg3/{M}x{N}x{K}"))
    return cases


def config4(n_shapes=2000, max_flops=2 ** 32, seed=None, config_index=4, prefix="cfg4"):
    """Random sweep for selector training and evaluation.

    M, N, K = round(2**(13 u)), u ~ U[0,1], drawn independently; the whole
    triple is redrawn while 2 M N K exceeds max_flops (rejection keeps the
    marginals log-uniform); transposes are fair coins; alpha ~ U[0.5, 2]; beta
    is 0, 1 or U[-1, 1] with probability 1/3 each.  Returns the cases in the
    shuffled order used for the 80/20 split (`split_train_heldout`).
    """
    rng = np.random.Generator(np.random.PCG64(case_seed(config_index, 0) if seed is None else seed))
    cases = []
    while len(cases) < n_shapes:
        dims = [int(round(2.0 ** (13.0 * rng.uniform()))) for _ in range(3)]
        dims = [min(max(d, 1), 8192) for d in dims]
        if 2 * dims[0] * dims[1] * dims[2] > max_flops:
            continue
        ta = TRANS if rng.uniform() < 0.5 else NO_TRANS
        tb = TRANS if rng.uniform() < 0.5 else NO_TRANS
        alpha = float(np.float32(rng.uniform(0.5, 2.0)))
        which = int(rng.integers(0, 3))
        beta_draw = float(np.float32(rng.uniform(-1.0, 1.0)))
        beta = (0.0, 1.0, beta_draw)[which]
        i = len(cases)
        cases.append(GemmCase(dims[0], dims[1], dims[2], ta, tb, alpha, beta, dist="uniform",
                              c0="uniform", seed=case_seed(config_index, i + 1), name=f"{prefix}/{i}"))
    order = rng.permutation(n_shapes)
    return [cases[i] for i in order]


def config_sweep2(n_shapes=4000):
    """A second random sweep drawn exactly like config4 from a stream of its own.  All of it trains (minus any
    shape that also occurs in an evaluation set): more inputs from the distribution the held-out shapes come from."""
    return config4(n_shapes, config_index=14, prefix="sweep2")


def config_sweep3(n_shapes=8000):
    """A third random sweep of the same recipe, again from a stream of its own; all of it trains."""
    return config4(n_shapes, config_index=17, prefix="sweep3")


def fresh_shapes(n_shapes, seed_index=0, log2_max_dim=13.0, max_flops=2 ** 32, min_work=0):
    """[n, 5] int64 rows (M, N, K, tA, tB) drawn like the random sweep (dimensions round(2**(log2_max_dim * u)),
    the triple redrawn while 2 M N K > max_flops or M N K < min_work, fair-coin transposes), from a stream of its
    own: shapes nobody has asked the selector about before, for timing its evaluation."""
    rng = np.random.Generator(np.random.PCG64(case_seed(40, seed_index)))
    rows = np.empty((0, 5), dtype=np.int64)
    while rows.shape[0] < n_shapes:
        d = np.rint(2.0 ** (log2_max_dim * rng.uniform(size=(2 * n_shapes, 3)))).astype(np.int64).clip(1, None)
        work = d[:, 0] * d[:, 1] * d[:, 2]
        d = d[(2 * work <= max_flops) & (work >= min_work)]
        t = rng.integers(0, 2, size=(d.shape[0], 2))
        rows = np.vstack([rows, np.column_stack([d, t])])
    return rows[:n_shapes]


def split_train_heldout(cases, train_fraction=0.8):
    """First 80 % of the (already shuffled) list trains, the rest is held out (Section 3, 'Datasets')."""
    n_train = int(round(train_fraction * len(cases)))
    return cases[:n_train], cases[n_train:]


def go2():
    """'Grid of two' triples (Section 4.1): every dimension from 256 to 3840 in steps of 256."""
    g = range(256, 3841, 256)
    return [(m, n, k) for m in g for n in g for k in g]


def po2():
    """'Power of two' triples (Section 4.1): every dimension a power of two from 64 to 2048."""
    g = [2 ** e for e in range(6, 12)]
    return [(m, n, k) for m in g for n in g for k in g]


def _dress(triples, config_index, prefix):
    """Triples -> cases with seeded transposes, alpha and beta drawn as in the random sweep."""
    rng = np.random.Generator(np.random.PCG64(case_seed(config_index, 0)))
    cases = []
    for i, (m, n, k) in enumerate(triples):
        ta = TRANS if rng.uniform() < 0.5 else NO_TRANS
        tb = TRANS if rng.uniform() < 0.5 else NO_TRANS
        alpha = float(np.float32(rng.uniform(0.5, 2.0)))
        which = int(rng.integers(0, 3))
        beta_draw = float(np.float32(rng.uniform(-1.0, 1.0)))
        cases.append(GemmCase(m, n, k, ta, tb, alpha, (0.0, 1.0, beta_draw)[which], dist="uniform", c0="uniform",
                              seed=case_seed(config_index, i + 1), name=f"{prefix}/{m}x{n}x{k}"))
    return cases


def config_go2():
    """The 'grid of two' triples of Section 4.1 as cases (transposes, alpha, beta seeded as in the random sweep)."""
    return _dress(go2(), 5, "go2")


def config_po2():
    """The 'power of two' triples of Section 4.1 as cases."""
    return _dress(po2(), 6, "po2")


def config_wide(n_shapes=1000, max_flops=2 ** 38, max_bytes=1.5e9, max_operand_bytes=6e8):
    """Wider random sweep: dimensions log-uniform in [1, 65536], rejected while the product exceeds
    max_flops, the operands together exceed max_bytes or one of them exceeds max_operand_bytes.  Covers the large and very rectangular corner (long
    convolution-lowered N, big squares) that the 2**32-flop cap of the main sweep leaves out."""
    rng = np.random.Generator(np.random.PCG64(case_seed(7, 0)))
    triples = []
    while len(triples) < n_shapes:
        m, n, k = (int(min(max(round(2.0 ** (16.0 * rng.uniform())), 1), 65536)) for _ in range(3))
        if 2 * m * n * k > max_flops or 4 * (m * k + k * n + m * n) > max_bytes:
            continue
        if 4 * max(m * k, k * n, m * n) > max_operand_bytes:
            continue
        triples.append((m, n, k))
    return _dress(triples, 7, "wide")


def config_big(n_shapes=200, max_flops=2 ** 41, max_bytes=1.5e9, max_operand_bytes=6e8):
    """Large products: dimensions log-uniform in [512, 16384] under the same memory caps as the wide sweep and
    2MNK <= max_flops.  Gives the selector training inputs in the range of the biggest square cases."""
    rng = np.random.Generator(np.random.PCG64(case_seed(8, 0)))
    triples = []
    while len(triples) < n_shapes:
        m, n, k = (int(round(512.0 * 2.0 ** (5.0 * rng.uniform()))) for _ in range(3))
        if 2 * m * n * k > max_flops or 4 * (m * k + k * n + m * n) > max_bytes:
            continue
        if 4 * max(m * k, k * n, m * n) > max_operand_bytes:
            continue
        triples.append((m, n, k))
    return _dress(triples, 8, "big")


def _log_uniform_sweep(config_index, prefix, n_shapes, m_range, n_range, k_range, max_flops=2 ** 38,
                       max_operand_bytes=6e8):
    rng = np.random.Generator(np.random.PCG64(case_seed(config_index, 0)))
    triples = []

    def draw(lo, hi):
        return int(round(lo * (hi / lo) ** rng.uniform()))

    while len(triples) < n_shapes:
        m, n, k = draw(*m_range), draw(*n_range), draw(*k_range)
        if 2 * m * n * k > max_flops or 4 * max(m * k, k * n, m * n) > max_operand_bytes:
            continue
        triples.append((m, n, k))
    return _dress(triples, config_index, prefix)


def config_thin(n_shapes=1000):
    """Thin products (few columns, many rows, long K): N in [1, 64], M in [256, 16384], K in [256, 8192],
    each log-uniform.  The region of fully-connected layers at small batch."""
    return _log_uniform_sweep(10, "thin", n_shapes, (256, 16384), (1, 64), (256, 8192))


def config_flat(n_shapes=1200):
    """Flat products (few rows, very many columns): M in [16, 512], N in [1024, 65536], K in [16, 4096],
    each log-uniform.  The region of convolutions lowered to GEMM."""
    return _log_uniform_sweep(11, "flat", n_shapes, (16, 512), (1024, 65536), (16, 4096))


def config_thin2(n_shapes=2000):
    """More of the thin corner, drawn like config_thin from a stream of its own."""
    return _log_uniform_sweep(15, "thin2", n_shapes, (256, 16384), (1, 64), (256, 8192))


def config_flat2(n_shapes=2000):
    """More of the flat corner, drawn like config_flat from a stream of its own."""
    return _log_uniform_sweep(16, "flat2", n_shapes, (16, 512), (1024, 65536), (16, 4096))


def config_thin3(n_shapes=2000):
    """A third draw of the thin corner."""
    return _log_uniform_sweep(18, "thin3", n_shapes, (256, 16384), (1, 64), (256, 8192))


def config_flat3(n_shapes=2000):
    """A third draw of the flat corner."""
    return _log_uniform_sweep(19, "flat3", n_shapes, (16, 512), (1024, 65536), (16, 4096))


def _geometric_grid(lo, hi):
    """Powers of two from lo to hi and the values half-way between them (3 * 2^e), ascending."""
    vals, v = [], lo
    while v <= hi:
        vals.append(v)
        if v >= 2 and v + v // 2 <= hi:
            vals.append(v + v // 2)
        v *= 2
    return vals


def config_thin_grid(max_flops=2 ** 38, max_operand_bytes=6e8):
    """Sparse geometric grid over the thin corner (a 'power of two' dataset in the sense of Section 4.1, moved to
    where fully-connected layers at small batch live): N a power of two up to 128, M and K powers of two and
    their midpoints.  Random sweeps almost never draw an N that is exactly 16 or 32, which is where the
    32-column tiles fit without waste; a grid does."""
    ns = [1, 2, 4, 8, 16, 32, 64, 128]
    triples = [(m, n, k) for m in _geometric_grid(256, 16384) for n in ns for k in _geometric_grid(256, 8192)
               if 2 * m * n * k <= max_flops and 4 * max(m * k, k * n, m * n) <= max_operand_bytes]
    return _dress(triples, 12, "tgrid")


def config_thin_grid2(max_flops=2 ** 38, max_operand_bytes=6e8):
    """A denser grid over the thin corner: N also at the midpoints (3, 6, 12, ...), M in quarter octaves from 512
    to 16384, K in half octaves from 512 to 8192; the triples config_thin_grid already holds are left out."""
    ns = [1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128]
    ms = sorted({(2 ** e) * q // 4 for e in range(9, 14) for q in (4, 5, 6, 7)} | {16384})
    have = {(c.M, c.N, c.K) for c in config_thin_grid(max_flops, max_operand_bytes)}
    triples = [(m, n, k) for m in ms for n in ns for k in _geometric_grid(512, 8192)
               if (m, n, k) not in have and 2 * m * n * k <= max_flops and 4 * max(m * k, k * n, m * n) <= max_operand_bytes]
    return _dress(triples, 20, "tgrid2")


def config_flat_grid(max_flops=2 ** 38, max_operand_bytes=6e8):
    """Sparse geometric grid over the flat corner (few rows, very many columns: convolutions lowered to GEMM):
    M a power of two from 16 to 512, N and K powers of two and their midpoints."""
    ms = [16, 32, 64, 128, 256, 512]
    triples = [(m, n, k) for m in ms for n in _geometric_grid(1024, 65536) for k in _geometric_grid(16, 4096)
               if 2 * m * n * k <= max_flops and 4 * max(m * k, k * n, m * n) <= max_operand_bytes]
    return _dress(triples, 13, "fgrid")


def config_large_grid(values=(2048, 3072, 4096, 6144, 8192, 12288), max_flops=2.5e12, max_bytes=1.5e9,
                      max_operand_bytes=6e8):
    """Coarse grid over the largest sizes one GPU call is asked for here (a 'grid' dataset in the sense of
    Section 4.1, at the top of the size range), under the same memory caps as the other sweeps."""
    triples = [(m, n, k) for m in values for n in values for k in values
               if 2 * m * n * k <= max_flops and 4 * (m * k + k * n + m * n) <= max_bytes
               and 4 * max(m * k, k * n, m * n) <= max_operand_bytes]
    return _dress(triples, 9, "large")


def bootstrap_indices(n_rows, n_trees, stream=0):
    """Seeded bootstrap samples for a forest of decision trees: n_trees arrays of n_rows row indices drawn with
    replacement.  Inputs of the training code and of the oracle alike (neither draws random numbers itself)."""
    return [np.random.Generator(np.random.PCG64(case_seed(20 + stream, t))).integers(0, n_rows, n_rows)
            for t in range(n_trees)]


# ------------------------------------------------------------------------------------------
# synthetic timing tables for selector tests (no GPU involved)
# ------------------------------------------------------------------------------------------

def synthetic_timing_table(n_shapes=400, n_variants=12, seed=7, noise=0.03, illegal_fraction=0.05):
    """A made-up but structured `shape x variant -> seconds` table for CPU tests of the selector.

    Each pretend variant has a tile size, a fixed launch cost and a rate; its
    time on a shape is launch + padded work / rate, times log-normal noise, and
    +inf where a made-up legality rule says it cannot run.  Variant 0 is legal
    everywhere (the universal fallback).  Returns (features [n,5] int64 with
    columns M, N, K, tA, tB; times [n, V] float64).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    feats = np.empty((n_shapes, 5), dtype=np.int64)
    feats[:, :3] = np.rint(2.0 ** (13.0 * rng.uniform(size=(n_shapes, 3)))).astype(np.int64).clip(1, 8192)
    feats[:, 3:] = rng.integers(0, 2, size=(n_shapes, 2))
    tile_m = 2 ** rng.integers(2, 9, size=n_variants)
    tile_n = 2 ** rng.integers(2, 9, size=n_variants)
    rate = 1e11 * (tile_m * tile_n) ** 0.5 * rng.uniform(0.7, 1.3, size=n_variants)
    launch = 4e-6 * rng.uniform(0.8, 2.0, size=n_variants)
    trans_pen = rng.uniform(0.9, 1.4, size=(n_variants, 2, 2))
    times = np.empty((n_shapes, n_variants), dtype=np.float64)
    for v in range(n_variants):
        M, N, K = feats[:, 0], feats[:, 1], feats[:, 2]
        pm = np.ceil(M / tile_m[v]) * tile_m[v]
        pn = np.ceil(N / tile_n[v]) * tile_n[v]
        waves = np.ceil(pm * pn / (tile_m[v] * tile_n[v]) / 256.0)
        work = waves * 256.0 * tile_m[v] * tile_n[v] * K * 2.0
        t = launch[v] + work / (rate[v] * 256.0)
        t = t * trans_pen[v, feats[:, 3], feats[:, 4]] * np.exp(noise * rng.standard_normal(n_shapes))
        times[:, v] = t
    illegal = rng.uniform(size=times.shape) < illegal_fraction
    illegal[:, 0] = False
    times[illegal] = np.inf
    return feats, times
