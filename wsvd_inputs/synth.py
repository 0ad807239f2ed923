from __future__ import annotations

import dataclasses
import numpy as np

__all__ = ["Spec", "SPECS", "spec", "rng", "normal", "bf16_exact", "outlier_sigma", "factors",
           "hidden_states", "latents_from_law", "ragged_lengths", "dense_wq", "int4_weight", "lowrank_q_factors",
           "norm_gains", "shared_up_factors", "shared_latents"]

# stream ids (second Philox key word)
_S_AK, _S_AV, _S_BK, _S_BV, _S_WQ, _S_X, _S_XNEW, _S_LAT, _S_LEN, _S_OUT, _S_W4, _S_WO, _S_AQ, _S_BQ, _S_GAIN, _S_SBK, _S_SBV, _S_SLAT = range(1, 19)


@dataclasses.dataclass(frozen=True)
class Spec:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    d_head: int
    d_model: int
    rank: int
    context: int            # rows already in the cache (max over the batch when ragged)
    latent_dtype: str       # "f32" | "bf16" | "i8" | "i4"
    factor_dtype: str       # "f32" | "bf16"
    q_dtype: str            # "f32" | "bf16" | "i8"
    ragged: tuple = ()      # (lo, hi) inclusive bounds of per-sequence lengths, or ()
    image_tokens: int = 0
    image_sigma: float = 1.0
    outlier_frac: float = 0.0
    outlier_gain: float = 20.0
    steps: int = 1          # consecutive decode steps
    layers: int = 1
    seed: int = 2604_02570


SPECS = {
    # the five workloads
    "c1": Spec("c1", 1, 8, 8, 64, 512, 16, 256, "f32", "f32", "f32"),
    "c2": Spec("c2", 1, 32, 32, 128, 4096, 32, 640, "bf16", "bf16", "bf16", image_tokens=576, image_sigma=1.5, steps=32),
    "c3": Spec("c3", 16, 32, 32, 128, 4096, 32, 2048, "i8", "bf16", "i8", outlier_frac=0.01),
    "c4": Spec("c4", 64, 32, 32, 128, 4096, 32, 4096, "i4", "bf16", "i8", ragged=(1024, 4096), image_tokens=576,
               image_sigma=1.5, outlier_frac=0.01),
    "c5": Spec("c5", 32, 28, 4, 128, 3584, 64, 8192, "i8", "bf16", "f32", outlier_frac=0.01, layers=28),
    # reduced shapes the fp64 oracle finishes in seconds; they still span several 64-row tiles and a ragged tail
    "c3_small": Spec("c3_small", 3, 4, 4, 128, 512, 32, 333, "i8", "bf16", "i8", outlier_frac=0.01),
    "c4_small": Spec("c4_small", 5, 4, 4, 128, 512, 32, 700, "i4", "bf16", "i8", ragged=(1, 700), image_tokens=100,
                     image_sigma=1.5, outlier_frac=0.01),
    "c5_small": Spec("c5_small", 3, 14, 2, 128, 512, 64, 300, "i8", "bf16", "f32", outlier_frac=0.01, layers=2),
    "c2_small": Spec("c2_small", 2, 4, 4, 128, 512, 32, 150, "bf16", "bf16", "bf16", image_tokens=100, image_sigma=1.5, steps=5),
}


def spec(name: str, **over) -> Spec:
    return dataclasses.replace(SPECS[name], **over) if over else SPECS[name]


def rng(seed: int, stream: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream * 1_000_003 + sub)]))


def normal(seed, stream, shape, sigma=1.0, sub=0) -> np.ndarray:
    return (rng(seed, stream, sub).standard_normal(shape, dtype=np.float32) * np.float32(sigma)).astype(np.float32)


def bf16_exact(x32: np.ndarray) -> np.ndarray:
    """Clear the low 16 mantissa bits so the fp32 value is exactly representable in bf16
    (a draw from a marginally different law, not a rounding rule of the method)."""
    u = np.ascontiguousarray(x32, np.float32).view(np.uint32) & np.uint32(0xFFFF0000)
    return u.view(np.float32)


def _as_dtype(x32, dtype):
    return bf16_exact(x32) if dtype == "bf16" else x32


def outlier_sigma(sp: Spec) -> np.ndarray:
    """Per-channel std of the hidden state: 1, except a fixed outlier_frac of channels at outlier_gain."""
    sig = np.ones(sp.d_model, np.float32)
    k = int(round(sp.outlier_frac * sp.d_model))
    if k:
        idx = rng(sp.seed, _S_OUT).choice(sp.d_model, size=k, replace=False)
        sig[idx] = sp.outlier_gain
    return sig


def factors(sp: Spec, layer: int = 0):
    """A_K, A_V [Hkv,E,r] ~ N(0,1/E); B_K, B_V [Hkv,r,d] ~ N(0,1/r); fp32 arrays (bf16-exact when factor_dtype is bf16)."""
    E, r, d, H = sp.d_model, sp.rank, sp.d_head, sp.n_kv_heads
    AK = _as_dtype(normal(sp.seed, _S_AK, (H, E, r), E ** -0.5, layer), sp.factor_dtype)
    AV = _as_dtype(normal(sp.seed, _S_AV, (H, E, r), E ** -0.5, layer), sp.factor_dtype)
    BK = _as_dtype(normal(sp.seed, _S_BK, (H, r, d), r ** -0.5, layer), sp.factor_dtype)
    BV = _as_dtype(normal(sp.seed, _S_BV, (H, r, d), r ** -0.5, layer), sp.factor_dtype)
    return AK, AV, BK, BV


def hidden_states(sp: Spec, n: int, sigma=1.0, which="new", sub=0, dtype=None) -> np.ndarray:
    """[n,E] hidden states ~ N(0, sigma^2 * diag(outlier_sigma^2))."""
    x = normal(sp.seed, _S_XNEW if which == "new" else _S_X, (n, sp.d_model), sigma, sub) * outlier_sigma(sp)[None, :]
    return _as_dtype(x.astype(np.float32), dtype or ("bf16" if sp.factor_dtype == "bf16" else "f32"))


def ragged_lengths(sp: Spec) -> np.ndarray:
    if not sp.ragged:
        return np.full(sp.batch, sp.context, np.int32)
    lo, hi = sp.ragged
    n = rng(sp.seed, _S_LEN).integers(lo, hi + 1, size=sp.batch).astype(np.int32)
    return n


def latents_from_law(sp: Spec, A: np.ndarray, which: str, b: int, n_rows: int, layer: int = 0) -> np.ndarray:
    """Latent rows of one sequence drawn from the law they would have if n_rows hidden states
    x_t ~ N(0, D) were pushed through the factor: c_t ~ N(0, A_h^T D A_h), D = diag(sigma_e^2),
    with the first image_tokens rows scaled by image_sigma.  Returns fp32 [Hkv, n_rows, r].
    (Sampling from the law instead of materialising tens of thousands of hidden vectors; the cache
    contents are inputs of the decode step, not results of it.)"""
    sig2 = outlier_sigma(sp).astype(np.float64) ** 2
    H, E, r = A.shape
    sub = ((layer * 4099 + b) * 2 + (0 if which == "k" else 1))
    z = rng(sp.seed, _S_LAT, sub).standard_normal((H, n_rows, r), dtype=np.float32).astype(np.float64)
    out = np.empty((H, n_rows, r), np.float32)
    for h in range(H):
        Ah = A[h].astype(np.float64)
        cov = Ah.T @ (Ah * sig2[:, None])
        L = np.linalg.cholesky(cov + 1e-12 * np.eye(r))
        c = z[h] @ L.T
        if sp.image_tokens:
            c[: min(sp.image_tokens, n_rows)] *= sp.image_sigma
        out[h] = c.astype(np.float32)
    return out


def dense_wq(sp: Spec) -> np.ndarray:
    """W_Q [E, Hq*d] ~ N(0,1/E), fp32."""
    return normal(sp.seed, _S_WQ, (sp.d_model, sp.n_q_heads * sp.d_head), sp.d_model ** -0.5)


def int4_weight(sp: Spec, n_out: int, which: int, layer: int = 0):
    """An int4-coded weight as the offline quantiser would leave it: codes [n_out, E] in [-8,7]
    (rounded Gaussian, std 2.5 codes) and a positive fp16 scale per output channel chosen so that
    code*scale has std ~ E^-1/2."""
    g = rng(sp.seed, _S_W4, layer * 16 + which)
    codes = np.clip(np.rint(g.standard_normal((n_out, sp.d_model), dtype=np.float32) * 2.5), -8, 7).astype(np.int8)
    scale = ((sp.d_model ** -0.5) / 2.5 * (0.75 + 0.5 * g.random(n_out, dtype=np.float32))).astype(np.float16)
    return codes, scale


def lowrank_q_factors(sp: Spec, rq: int, layer: int = 0):
    """Per-head low-rank query factors: A_Q [Hq,E,rq] ~ N(0,1/E) and B_Q [Hq,rq,d] ~ N(0,1/rq), fp32 (B_Q bf16-exact when
    the factors are bf16), so that q = x A_Q B_Q has unit-variance entries like the dense query."""
    AQ = normal(sp.seed, _S_AQ, (sp.n_q_heads, sp.d_model, rq), sp.d_model ** -0.5, sub=layer)
    BQ = normal(sp.seed, _S_BQ, (sp.n_q_heads, rq, sp.d_head), rq ** -0.5, sub=layer)
    return AQ, _as_dtype(BQ, sp.factor_dtype)


def norm_gains(sp: Spec, which: int, layer: int = 0) -> np.ndarray:
    """RMSNorm gain [E] = 1 + 0.1 N(0,1), fp32."""
    return (1.0 + normal(sp.seed, _S_GAIN, (sp.d_model,), 0.1, sub=layer * 4 + which)).astype(np.float32)


def shared_up_factors(sp: Spec, R: int, layer: int = 0):
    """Up-projection factors of the whole-matrix scheme: every head has its own B_Kh, B_Vh [R, d] over ONE shared latent
    of rank R.  B_K, B_V [Hq, R, d] ~ N(0, 1/R), bf16-exact fp32."""
    H, d = sp.n_q_heads, sp.d_head
    BK = bf16_exact(normal(sp.seed, _S_SBK, (H, R, d), R ** -0.5, layer))
    BV = bf16_exact(normal(sp.seed, _S_SBV, (H, R, d), R ** -0.5, layer))
    return BK, BV


def shared_latents(sp: Spec, R: int, which: str, b: int, n_rows: int, layer: int = 0) -> np.ndarray:
    """Rows of the shared latent of one sequence, fp32 [n_rows, R]: unit-variance Gaussians with the per-channel spread
    of the outlier profile (a few channels much wider than the rest) and the image-token prefix scaled like the
    per-head recipe's."""
    g = rng(sp.seed, _S_SLAT, (layer * 2 + (0 if which == "k" else 1)) * 4096 + b)
    c = g.standard_normal((n_rows, R), dtype=np.float32)
    prof = outlier_sigma(sp)
    c *= np.resize(prof, R).astype(np.float32)[None, :]
    n_img = min(n_rows, int(getattr(sp, "image_tokens", 0)))
    if n_img:
        c[:n_img] *= np.float32(getattr(sp, "image_sigma", 1.0))
    return c
