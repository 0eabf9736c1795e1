"""Seeded synthetic inputs shared by the GPU path's tests, the oracle's tests and the benchmark.

This module only draws random tensors and describes the benchmark workloads; it holds none of
the contraction arithmetic and imports neither the GPU binding nor the oracle.

The paper measures on randomised dense tensors (section IV), mostly cubic n x n x n; the
workloads below follow that recipe: dense, column-major packed, entries uniform in [-1, 1]
(normal(0,1) rounded to bf16 for the bf16 workload), drawn from numpy's PCG64 generator.
"""
import numpy as np

BASE_SEED = 160605696


def seed_for(cfg: int, which: str) -> int:
    """Seed of tensor `which` ('A', 'B' or 'C') of workload number `cfg`."""
    return BASE_SEED + 10 * int(cfg) + {"A": 0, "B": 1, "C": 2}[which]


def uniform_tensor(seed: int, dims, dtype=np.float64) -> np.ndarray:
    """Column-major array of the given logical shape with entries uniform in [-1, 1]."""
    rng = np.random.default_rng(seed)
    n = int(np.prod(dims, dtype=np.int64)) if len(dims) else 1
    flat = rng.uniform(-1.0, 1.0, size=n).astype(dtype)
    return flat.reshape(tuple(dims), order="F")


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result is fp32 holding bf16 values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    rounded = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    nan = np.isnan(x)
    out = rounded.astype(np.uint32).view(np.float32).reshape(x.shape)
    if nan.any():
        out = np.where(nan, np.float32(np.nan), out)
    return out


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """The 16-bit patterns of fp32 values that are already exact bf16 numbers."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def bf16_from_bits(bits: np.ndarray) -> np.ndarray:
    """fp32 values of 16-bit bf16 patterns."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return b.view(np.float32).reshape(bits.shape)


def normal_bf16_tensor(seed: int, dims) -> np.ndarray:
    """Column-major fp32 array of normal(0,1) draws, each rounded to bf16."""
    rng = np.random.default_rng(seed)
    n = int(np.prod(dims, dtype=np.int64)) if len(dims) else 1
    flat = round_to_bf16(rng.standard_normal(size=n).astype(np.float32))
    return flat.reshape(tuple(dims), order="F")


def make_tensor(seed: int, dims, dtype: str) -> np.ndarray:
    """Input tensor for element type 'f64', 'f32' (uniform) or 'bf16' (normal, bf16-exact fp32)."""
    if dtype == "f64":
        return uniform_tensor(seed, dims, np.float64)
    if dtype == "f32":
        return uniform_tensor(seed, dims, np.float32)
    if dtype == "bf16":
        return normal_bf16_tensor(seed, dims)
    raise ValueError("unknown dtype %r" % dtype)


# The benchmark workloads: mode strings, extents per index, element type, and the
# evaluation the workload names (annotated in the paper's batching / flattening notation).
WORKLOADS = {
    # small reference case the oracle finishes at once
    1: dict(name="cfg1: C_mnp = A_mk B_knp, 32^4, f64, SBGEMM [p]",
            A="mk", B="knp", C="mnp", ext=dict(m=32, n=32, p=32, k=32), dtype="f64",
            eval=("mk", "kn[p]", "mn[p]")),
    # tiny-batch regime
    3: dict(name="cfg3: C_mnp = A_mk B_knp, m=n=k=16, p=65536, f32, SBGEMM [p]",
            A="mk", B="knp", C="mnp", ext=dict(m=16, n=16, p=65536, k=16), dtype="f32",
            eval=("mk", "kn[p]", "mn[p]")),
    # large cube, A transposed, batch over p
    40: dict(name="cfg4a: C_mnp = A_km B_knp, 512^4, f64, SBGEMM [p]",
             A="km", B="knp", C="mnp", ext=dict(m=512, n=512, p=512, k=512), dtype="f64",
             eval=("km", "kn[p]", "mn[p]")),
    41: dict(name="cfg4b: C_mnp = A_km B_knp, 512^4, f32, SBGEMM [p]",
             A="km", B="knp", C="mnp", ext=dict(m=512, n=512, p=512, k=512), dtype="f32",
             eval=("km", "kn[p]", "mn[p]")),
    # order-3 x order-3, nested batching over (p, q)
    5: dict(name="cfg5: C_mpnq = A_mpk B_knq, m=n=p=q=64, k=128, bf16, nested [p][q]",
            A="mpk", B="knq", C="mpnq", ext=dict(m=64, n=64, p=64, q=64, k=128), dtype="bf16",
            eval=("m[p]k", "kn[q]", "m[p]n[q]")),
}


def workload_tensors(cfg: int, with_c: bool = False):
    """(A, B[, C_old]) of workload `cfg` as column-major numpy arrays of logical shape."""
    w = WORKLOADS[cfg]
    seed_cfg = {40: 4, 41: 4}.get(cfg, cfg)
    dA = [w["ext"][c] for c in w["A"]]
    dB = [w["ext"][c] for c in w["B"]]
    out = [make_tensor(seed_for(seed_cfg, "A"), dA, w["dtype"]),
           make_tensor(seed_for(seed_cfg, "B"), dB, w["dtype"])]
    if with_c:
        dC = [w["ext"][c] for c in w["C"]]
        out.append(make_tensor(seed_for(seed_cfg, "C"), dC, w["dtype"]))
    return tuple(out)


def lowrank_noise_tensor(seed: int, dims, core, noise: float = 0.05, dtype=np.float64) -> np.ndarray:
    """Synthetic input for the Tucker application study (section IV-C works on cubic tensors with a
    10 x 10 x 10 core): a random core of size `core` with decaying entries, expanded by random
    orthonormal factors to `dims`, plus uniform noise of relative size `noise`.  Column-major."""
    rng = np.random.default_rng(seed)
    G = rng.standard_normal(core)
    for r, c in enumerate(core):                       # decaying weights: distinct, well-separated singular values
        w = 1.0 / (1.0 + np.arange(c))
        G = G * w.reshape([-1 if a == r else 1 for a in range(3)])
    factors = [np.linalg.qr(rng.standard_normal((d, c)))[0] for d, c in zip(dims, core)]
    T = G                                              # mode products one at a time (T = G x1 F0 x2 F1 x3 F2)
    for r, F in enumerate(factors):
        T = np.moveaxis(np.tensordot(F, T, axes=(1, r)), 0, r)
    T = T / np.sqrt(np.mean(T * T))
    T = T + noise * rng.uniform(-1.0, 1.0, size=T.shape)
    return np.asfortranarray(T.astype(dtype))
