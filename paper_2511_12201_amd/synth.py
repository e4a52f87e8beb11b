"""Seeded synthetic inputs with the shape of long-video attention workloads.

This module serves both the HIP path's tests/benchmark and the CPU oracle's
tests.  It holds none of the method's arithmetic: it only draws tensors.

The paper evaluates on video benchmarks with trained 7B models; neither the
data nor the weights are available, so inputs are drawn from a generator that
takes the paper's shapes (frames x tokens-per-frame visual tokens followed by a
short text segment; 28 query / 4 KV heads of dimension 128 for the 7B backbone)
and its reported structure (Sec. "Introduction", Fig. 1: most queries look at
the attention sink or at spatio-temporally adjacent tokens, a minority look
broadly; heads differ in sharpness).

Recipe (all draws from numpy's PCG64 seeded with `seed`):
  * Q, K, V ~ N(0, 1) i.i.d.
  * per (KV head, frame) a cluster mean c ~ N(0, 0.5 I) is added to the keys of
    that frame and to the queries of that frame in the heads of the group, so
    attention concentrates within frames; text tokens get none.
  * structured configurations add three things.  (a) A random-Fourier positional
    code phi(n) (phi(n).phi(m) ~ exp(-(n-m)^2 / 2 W^2), W = 64) on every key
    with gain beta (beta^2 / sqrt(d) = 6): a local window.  (b) A bounded key
    salience: K[n] += gamma s_n w with s_n ~ U[-1, 1] (0 at the sink), w a unit
    direction per KV head orthogonal to the sink key, and every query carries
    gamma w (gamma^2 / sqrt(d) = 8.4), so a head's accumulated key scores are
    roughly log-uniform with a spread that grows with the head's sharpness,
    which keeps the kurtosis ordering of heads tied to their budget need.
    (c) Each visual query is "lazy" with probability 0.7 and then becomes
    0.25 q + lambda u_sink + beta phi(n), where u_sink is the unit sink key and
    lambda puts the sink logit at +5; the other queries stay broad.  Finally
    the queries of head i are multiplied by t_i: t_0 = 0.5 and t_1..t_{H-1} on a
    geometric ramp 1.3 .. 3, so head 0 is clearly the flattest by design.
    `plain` leaves out (b) and puts all heads on one ramp 0.5 .. 2: the first form of the recipe, on which the
    kurtosis arg-min is decided by outliers; the benchmark reports both.
  * bf16 configurations round Q, K, V to the bf16 grid (nearest-even); arrays
    stay float32 so the oracle reads exactly the values the GPU reads.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class LayerCfg:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    frames: int
    tok_per_frame: int
    n_text: int
    dtype: str            # "f32" or "bf16"
    structured: bool
    seed: int
    causal: bool = True
    plain: bool = False   # structured configurations only: leave out the key salience (b) and put the heads' sharpness
                          # on one geometric ramp 0.5 .. 2 -- the configuration text's generator without the two
                          # additions that tie the kurtosis order of the heads to their budget need

    @property
    def n_vis(self) -> int:
        return self.frames * self.tok_per_frame

    @property
    def n_tokens(self) -> int:
        return self.n_vis + self.n_text

    @property
    def vis_begin(self) -> int:
        return 0

    @property
    def vis_end(self) -> int:
        return self.n_vis

    @property
    def sink_index(self) -> int:
        return 0

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))

    def scaled(self, **kw) -> "LayerCfg":
        return replace(self, **kw)


# The five workloads named by the build's baseline description.
C1_TINY = LayerCfg("c1_tiny", 1, 2, 2, 64, 4, 240, 64, "f32", False, 0)
C2_16K = LayerCfg("c2_16k", 1, 28, 4, 128, 64, 252, 256, "bf16", True, 1)
C3_64K = LayerCfg("c3_64k", 1, 28, 4, 128, 256, 252, 1024, "bf16", True, 2)
C4_TRAIN_32K = LayerCfg("c4_train_32k", 1, 28, 4, 128, 128, 252, 512, "bf16", True, 3)
C5_DECODE_131K = LayerCfg("c5_decode_131k", 1, 28, 4, 128, 512, 252, 2048, "bf16", True, 4)

LAZY_FRACTION = 0.7
WINDOW = 64.0
SINK_LOGIT = 5.0
LOCAL_GAIN = 6.0          # beta^2 / sqrt(d)
CLUSTER_VAR = 0.5
SHARP_FLAT, SHARP_LO, SHARP_HI = 0.5, 1.3, 3.0
SALIENCE_GAIN = 8.4       # gamma^2 / sqrt(d)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that already lie on the bf16 grid (int16 view)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16).view(np.int16)


def _positional_code(rng, n_tokens: int, d: int) -> np.ndarray:
    omega = rng.standard_normal(d) / WINDOW
    theta = rng.uniform(0.0, 2.0 * np.pi, d)
    n = np.arange(n_tokens, dtype=np.float64)[:, None]
    return (np.sqrt(2.0 / d) * np.cos(n * omega[None, :] + theta[None, :])).astype(np.float32)


def head_sharpness(n_q_heads: int, plain: bool = False) -> np.ndarray:
    if n_q_heads == 1:
        return np.ones(1, dtype=np.float32)
    if plain:
        i = np.arange(n_q_heads, dtype=np.float64)
        return (0.5 * 4.0 ** (i / (n_q_heads - 1))).astype(np.float32)
    i = np.arange(n_q_heads - 1, dtype=np.float64)
    ramp = SHARP_LO * (SHARP_HI / SHARP_LO) ** (i / max(1, n_q_heads - 2))
    return np.concatenate([[SHARP_FLAT], ramp]).astype(np.float32)


def _lazy_transform(q, u_sink, lam, beta, phi_rows):
    return 0.25 * q + (lam * u_sink)[None, :] + beta * phi_rows


def make_layer(cfg: LayerCfg):
    """Returns dict(Q [B,Hq,N,d], K, V [B,Hkv,N,d]) float32 plus generator side data
    needed to draw matching decode queries (positional code, gains)."""
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    B, Hq, Hkv, d, N = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.n_tokens
    G = Hq // Hkv
    F, T = cfg.frames, cfg.tok_per_frame
    Q = rng.standard_normal((B, Hq, N, d), dtype=np.float32)
    K = rng.standard_normal((B, Hkv, N, d), dtype=np.float32)
    V = rng.standard_normal((B, Hkv, N, d), dtype=np.float32)
    centres = (np.sqrt(CLUSTER_VAR) * rng.standard_normal((B, Hkv, F, d))).astype(np.float32)
    per_tok = np.repeat(centres, T, axis=2)                       # [B,Hkv,N_v,d]
    K[:, :, : F * T] += per_tok
    for i in range(Hq):
        Q[:, i, : F * T] += per_tok[:, i // G]
    side = dict(beta=0.0, phi=None, lam=None, u_sink=None, sharp=np.ones(Hq, dtype=np.float32))
    if cfg.structured:
        beta = float(np.sqrt(LOCAL_GAIN * np.sqrt(d)))
        phi = _positional_code(rng, N, d)
        K += beta * phi[None, None]
        ks = K[:, :, cfg.sink_index, :].astype(np.float64)
        norm = np.linalg.norm(ks, axis=-1, keepdims=True)
        u_sink = (ks / norm).astype(np.float32)                      # [B,Hkv,d]
        lam = (SINK_LOGIT * np.sqrt(d) / norm[..., 0]).astype(np.float32)
        if not cfg.plain:
            gamma = float(np.sqrt(SALIENCE_GAIN * np.sqrt(d)))
            w = rng.standard_normal((B, Hkv, d))
            w -= (w * u_sink).sum(axis=-1, keepdims=True) * u_sink    # salience direction is orthogonal to the sink key
            w = (w / np.linalg.norm(w, axis=-1, keepdims=True)).astype(np.float32)
            sal = rng.uniform(-1.0, 1.0, (B, Hkv, N)).astype(np.float32)
            sal[:, :, cfg.sink_index] = 0.0
            K += gamma * sal[..., None] * w[:, :, None, :]
            for i in range(Hq):
                Q[:, i] += gamma * w[:, i // G, None, :]
        lazy = rng.random((B, Hq, F * T)) < LAZY_FRACTION
        sharp = head_sharpness(Hq, cfg.plain)
        for b in range(B):
            for i in range(Hq):
                g = i // G
                rows = np.nonzero(lazy[b, i])[0]
                Q[b, i, rows] = _lazy_transform(Q[b, i, rows], u_sink[b, g], lam[b, g], beta, phi[rows])
                Q[b, i] *= sharp[i]
        side = dict(beta=beta, phi=phi, lam=lam, u_sink=u_sink, sharp=sharp)
    if cfg.dtype == "bf16":
        Q, K, V = round_to_bf16(Q), round_to_bf16(K), round_to_bf16(V)
    return dict(Q=Q, K=K, V=V, side=side)


def make_grad_output(cfg: LayerCfg):
    """dO ~ N(0,1)/sqrt(d), rounded like the layer's dtype.  [B,Hq,N,d] float32."""
    rng = np.random.Generator(np.random.PCG64(cfg.seed + 1000))
    dO = rng.standard_normal((cfg.batch, cfg.n_q_heads, cfg.n_tokens, cfg.head_dim), dtype=np.float32)
    dO *= np.float32(cfg.scale)
    return round_to_bf16(dO) if cfg.dtype == "bf16" else dO


def make_decode_steps(cfg: LayerCfg, layer, n_steps: int, batch: int | None = None):
    """Decode-phase tensors for `n_steps` new tokens after a prefill of cfg.n_tokens.

    Returns dict(q [S,B,Hq,d], k_new, v_new [S,B,Hkv,d]) float32.  Each step's
    query follows the prefill mixture: lazy with probability 0.7 per head (then
    pulled towards the sink key), otherwise broad.  `batch` > cfg.batch repeats
    the draw with independent noise for the extra sequences, reusing the side
    data of sequence b % cfg.batch.
    """
    B = cfg.batch if batch is None else batch
    rng = np.random.Generator(np.random.PCG64(cfg.seed + 2000))
    Hq, Hkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    G = Hq // Hkv
    side = layer["side"]
    q = rng.standard_normal((n_steps, B, Hq, d), dtype=np.float32)
    k_new = rng.standard_normal((n_steps, B, Hkv, d), dtype=np.float32)
    v_new = rng.standard_normal((n_steps, B, Hkv, d), dtype=np.float32)
    if cfg.structured:
        lazy = rng.random((n_steps, B, Hq)) < LAZY_FRACTION
        for s in range(n_steps):
            for b in range(B):
                sb = b % cfg.batch
                for i in range(Hq):
                    if lazy[s, b, i]:
                        q[s, b, i] = 0.25 * q[s, b, i] + side["lam"][sb, i // G] * side["u_sink"][sb, i // G]
                    q[s, b, i] *= side["sharp"][i]
    if cfg.dtype == "bf16":
        q, k_new, v_new = round_to_bf16(q), round_to_bf16(k_new), round_to_bf16(v_new)
    return dict(q=q, k_new=k_new, v_new=v_new)
