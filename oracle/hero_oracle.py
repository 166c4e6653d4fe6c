"""CPU oracle for HERO's cached DiT denoising step -- TEST INFRASTRUCTURE ONLY.

A plain, slow, by-the-definitions implementation in numpy (float64 unless a
dtype is passed) of what the hot path computes.  It exists so the HIP path can
be checked against something written independently from the paper; it is not a
product path and shares no code with the HIP library (the only common import is
the seeded input generator, which holds no method arithmetic).  Only tests,
the smoke check and the benchmark's cpu_baseline leg may import it.

HERO is an approximation scheme, so the oracle takes the algorithm's steps in
the paper's order and notation:

  block             Eq. 2 (Sec. 3.2): G, H = F(LN(z, tau)); z, tau += G, H for
                    F in {FullAttn, FFN}; scale/shift omitted as the paper does.
  full_layer        Alg. 1 "Initial Caching": run the block on all rows, store
                    G (attention branch) and G (FFN branch); shallow layers also
                    keep K, V of every row; deep layers keep the previous
                    generation so that Delta G = G_t - G_{t+M} is available.
  refresh_layer     Eq. 3 / Alg. 1 (l < K): recompute F on the selected rows
                    only, against the full cached K/V, merge into the cache.
  extrapolate_layer Eq. 5 / Alg. 1 (l >= K): G_{t-k} = G_t + (G_t - G_{t+M}) k/M
                    followed by the plain residual add.
  select            Eq. 4 (patch-wise sampling) with the frequency-aware
                    tracking paragraph of Sec. 3.3.
  HeroOracle.step   Alg. 1's outer loops.
  second_difference_variance / stability_scores
                    the per-layer stability score of Sec. 3.2's feature analysis.

Readings taken where the paper is silent or inconsistent (each is listed in
the design notes at the repository root):
  * layers are 0-indexed, l < K refresh, l >= K extrapolate;
  * a full step happens when step % M == 0, cached steps have k = 1..M-1;
  * Delta G = 0 until two full-step generations exist;
  * refreshed K/V rows are written to the cache before attention and the
    refreshed queries attend to all N cached keys (text + video, no mask);
  * refreshed features are merged into the cache in place (a later cached step
    reuses the most recent value of a row);
  * text rows are never selected; they reuse their cached features;
  * tokens per patch n_p = clamp(floor(R*|patch| + 1/2), 1, |patch|), edge
    patches are clipped to the grid and sized on their own;
  * Sample(P, R) is deterministic age-priority: within a patch take the n_p
    tokens with the largest (age, hash) key, hash = mix32(seed, step, token);
    a second, stochastic reading (select_mode 1) draws the n_p tokens without
    replacement with probability proportional to age + 1;
  * stability score: population variance of F_{t+1} - 2 F_t + F_{t-1} over all
    elements and steps, then 1 - (v - min) / (max - min) across layers;
    selected ages become 0, all others grow by 1, a full step zeroes all ages;
  * the block is pre-LayerNorm with affine parameters, biased Linear layers,
    tanh-form GELU and softmax scale 1/sqrt(head_dim).

Parity status: every function here is pinned by tests/test_oracle_*.py against
closed forms, brute force, library routines, enumerated probabilities or
invariants.  Parity unpinned (the paper gives no formula; the invariants are
pinned, the particular choice is this repository's reading): which tokens a
patch yields under either sampling rule; the normalisation of the stability
score (min-max, inverted); the composition of the modulated block (where the
gate sits, which stream a row belongs to, the rotary channel split), whose
pieces are each pinned against their textbook definitions.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Tuple

import numpy as np

# ----------------------------------------------------------------------------
# block components (Eq. 2, with the internals the paper omits "for clarity")
# ----------------------------------------------------------------------------


def layer_norm(x: np.ndarray, gain: np.ndarray, bias: np.ndarray, eps: float) -> np.ndarray:
    """LayerNorm over the last axis: (x - mean) / sqrt(var + eps) * gain + bias (Eq. 2's LN)."""
    mean = x.mean(axis=-1, keepdims=True)
    var = ((x - mean) ** 2).mean(axis=-1, keepdims=True)
    return (x - mean) / np.sqrt(var + eps) * gain + bias


def gelu_tanh(x: np.ndarray) -> np.ndarray:
    """GELU, tanh form: x/2 * (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3)))."""
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def linear(x: np.ndarray, w: np.ndarray, b: np.ndarray) -> np.ndarray:
    """y = x W^T + b with W stored [out_features, in_features]."""
    return x @ w.T + b


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, n_heads: int) -> np.ndarray:
    """softmax(q_h k_h^T / sqrt(hd)) v_h per head h, heads concatenated (FullAttn in Eq. 2).

    q: [r, d], k, v: [N, d]; every query attends to all N keys, no mask.
    """
    r, d = q.shape
    hd = d // n_heads
    out = np.empty_like(q)
    for h in range(n_heads):
        sl = slice(h * hd, (h + 1) * hd)
        s = (q[:, sl] @ k[:, sl].T) / math.sqrt(hd)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p /= p.sum(axis=1, keepdims=True)
        out[:, sl] = p @ v[:, sl]
    return out


def ffn(u: np.ndarray, w: Dict[str, np.ndarray]) -> np.ndarray:
    """FFN in Eq. 2: GELU(u W1^T + b1) W2^T + b2."""
    return linear(gelu_tanh(linear(u, w["w_ff1"], w["b_ff1"])), w["w_ff2"], w["b_ff2"])


def _cast_weights(w: Dict[str, np.ndarray], dtype) -> Dict[str, np.ndarray]:
    return {k: np.asarray(v, dtype=dtype) for k, v in w.items()}


# ----------------------------------------------------------------------------
# selection (Eq. 4 + frequency-aware tracking)
# ----------------------------------------------------------------------------

_M32 = 0xFFFFFFFF


def fmix32(h: np.ndarray) -> np.ndarray:
    """32-bit avalanche finaliser (xor-shift / odd multiply, three shifts, two multiplies)."""
    h = np.asarray(h, dtype=np.uint64) & _M32
    h ^= h >> np.uint64(16)
    h = (h * np.uint64(0x85EBCA6B)) & _M32
    h ^= h >> np.uint64(13)
    h = (h * np.uint64(0xC2B2AE35)) & _M32
    h ^= h >> np.uint64(16)
    return h


def mix32(seed: int, step: int, token: np.ndarray) -> np.ndarray:
    """Per-(seed, step, token) 32-bit hash used as the random tie-break among equal ages.

    s0 = lo32(seed) xor hi32(seed); s1 = fmix32(s0 + 0x9E3779B9 * (step + 1));
    hash = fmix32(s1 xor (token * 0x85EBCA6B)), all modulo 2^32.  For a fixed
    step distinct tokens get distinct hashes (every stage is a bijection).
    """
    s0 = ((seed & _M32) ^ ((seed >> 32) & _M32)) & _M32
    s1 = int(fmix32(np.uint64((s0 + 0x9E3779B9 * ((step + 1) & _M32)) & _M32)))
    t = (np.asarray(token, dtype=np.uint64) * np.uint64(0x85EBCA6B)) & _M32
    return fmix32(np.uint64(s1) ^ t)


def tokens_per_patch(ratio: float, size: int) -> int:
    """n_p = clamp(floor(R * |patch| + 1/2), 1, |patch|); 0 when R <= 0.

    R is taken at float32 precision (the precision the configuration carries it
    in); R * size + 1/2 is then exact in float64 for any realistic patch size.
    """
    r = float(np.float32(ratio))
    if r <= 0.0:
        return 0
    return int(min(max(math.floor(r * size + 0.5), 1), size))


def patch_list(frames: int, height: int, width: int, ph: int, pw: int
               ) -> List[Tuple[int, int, int, int, int]]:
    """Non-overlapping spatial patches per latent frame (Eq. 4), frame-major then
    patch-row then patch-column; edge patches are clipped to the grid.
    Each entry is (t, y0, x0, hh, ww)."""
    out = []
    for t in range(frames):
        for y0 in range(0, height, ph):
            for x0 in range(0, width, pw):
                out.append((t, y0, x0, min(ph, height - y0), min(pw, width - x0)))
    return out


SELECT_AGE_PRIORITY = 0     # deterministic: oldest first, hash breaks ties
SELECT_AGE_WEIGHTED = 1     # stochastic: sampling without replacement, probability ~ age + 1

AGE_WEIGHT_CAP = 0xFFFF     # weights are min(age, cap) + 1 so a patch's total stays below 2^32


def draw32(seed: int, step: int, first_token: int, draw: int) -> int:
    """32-bit random word of draw number `draw` (0-based) in the patch whose first
    (top-left) token is `first_token`: fmix32(mix32(seed, step, first_token) +
    0x9E3779B9 * (draw + 1)) modulo 2^32."""
    base = int(mix32(seed, step, np.array([first_token]))[0])
    return int(fmix32(np.uint64((base + 0x9E3779B9 * (draw + 1)) & _M32)))


def sample_weighted(weights: List[int], n_take: int, words: List[int]) -> List[int]:
    """Weighted sampling without replacement, one draw at a time (the textbook
    sequential scheme): with W the total weight of the items not yet taken, draw
    number j maps its 32-bit word u to r = floor(u * W / 2^32) in [0, W) and takes
    the first remaining item, in list order, whose running weight sum exceeds r.
    Returns the taken positions in draw order."""
    left = list(range(len(weights)))
    taken = []
    for j in range(n_take):
        total = sum(weights[e] for e in left)
        r = (words[j] * total) >> 32
        run = 0
        for e in left:
            run += weights[e]
            if run > r:
                taken.append(e)
                left.remove(e)
                break
    return taken


def select(ages: np.ndarray, cfg, step: int) -> Tuple[np.ndarray, np.ndarray]:
    """S(z) of Eq. 4 with the frequency-aware tracking of Sec. 3.3.

    ages: int32 [n_video] (how many cached steps each token has gone unsampled).
    Returns (idx, new_ages): idx are joint-sequence row indices (n_text + token),
    ordered patch-major.  Two readings of "higher sampling probabilities to those
    neglected longer", chosen by cfg.select_mode (default: age priority):
      age priority  -- inside a patch the n_p tokens with the largest (age, hash)
                       key, listed by decreasing key;
      age weighted  -- n_p draws without replacement with probability
                       proportional to age + 1 among the tokens still left
                       (tokens in row-major order inside the patch), listed in
                       draw order.
    """
    ages = np.asarray(ages, dtype=np.int64)
    mode = getattr(cfg, "select_mode", SELECT_AGE_PRIORITY)
    sel: List[int] = []
    for (t, y0, x0, hh, ww) in patch_list(cfg.frames, cfg.height, cfg.width, cfg.patch_h, cfg.patch_w):
        toks = np.array([(t * cfg.height + (y0 + dy)) * cfg.width + (x0 + dx)
                         for dy in range(hh) for dx in range(ww)], dtype=np.int64)
        n_p = tokens_per_patch(cfg.ratio, len(toks))
        if mode == SELECT_AGE_WEIGHTED:
            weights = [min(int(a), AGE_WEIGHT_CAP) + 1 for a in ages[toks]]
            words = [draw32(cfg.seed, step, int(toks[0]), j) for j in range(n_p)]
            sel.extend(int(toks[e]) for e in sample_weighted(weights, n_p, words))
            continue
        hashes = mix32(cfg.seed, step, toks).astype(np.int64)
        keys = (ages[toks] << 32) | hashes
        order = np.argsort(-keys, kind="stable")  # keys are distinct: hashes are
        sel.extend(int(toks[j]) for j in order[:n_p])
    sel_arr = np.array(sel, dtype=np.int64)
    new_ages = ages + 1
    new_ages[sel_arr] = 0
    return (sel_arr + cfg.n_text).astype(np.int32), new_ages.astype(np.int32)


# ----------------------------------------------------------------------------
# layer operations on a cache (Alg. 1)
# ----------------------------------------------------------------------------

# ----------------------------------------------------------------------------
# the modulated block: the internals Sec. 3.2 leaves out "for clarity" (scale and
# shift), as CogVideoX-style DiT blocks have them.  The paper fixes none of this;
# each piece is the textbook definition and is pinned as such by the tests.
# ----------------------------------------------------------------------------

BLOCK_ADALN, BLOCK_QKNORM, BLOCK_ROPE = 1, 2, 4
QK_NORM_EPS = 1e-6
ROPE_THETA = 10000.0
MOD_ROWS = ("shift1_v", "scale1_v", "gate1_v", "shift1_t", "scale1_t", "gate1_t",
            "shift2_v", "scale2_v", "gate2_v", "shift2_t", "scale2_t", "gate2_t")


def stream_vector(mod: np.ndarray, name: str, rows: np.ndarray, n_text: int) -> np.ndarray:
    """Per-row modulation vector: row `name`_t of the table for text rows
    (joint index < n_text), `name`_v for video rows.  -> [len(rows), d]."""
    v = mod[MOD_ROWS.index(name + "_v")]
    t = mod[MOD_ROWS.index(name + "_t")]
    return np.where((np.asarray(rows) < n_text)[:, None], t[None, :], v[None, :])


def head_layer_norm(x: np.ndarray, gain: np.ndarray, bias: np.ndarray, n_heads: int) -> np.ndarray:
    """LayerNorm over each head's channels separately (q/k normalisation), eps 1e-6,
    one gain/bias vector [head_dim] shared by all heads."""
    r, d = x.shape
    xh = x.reshape(r, n_heads, d // n_heads)
    return layer_norm(xh, gain, bias, QK_NORM_EPS).reshape(r, d)


def rope_angles(frames: int, height: int, width: int, head_dim: int) -> np.ndarray:
    """Rotation angles of the 3-D rotary position embedding, [frames*height*width, head_dim/2].

    The head's channel pairs are split between the axes: head_dim/8 pairs for t,
    then 3*head_dim/16 pairs each for y and x (16 / 24 / 24 channels at head_dim
    64).  Pair i of an axis with n pairs turns by pos * theta^(-i/n), theta = 10000.
    Token order (t, y, x) row-major, as in the joint sequence."""
    n_t, n_y = head_dim // 8, (head_dim // 16) * 3
    n_x = head_dim // 2 - n_t - n_y
    t, y, x = np.meshgrid(np.arange(frames), np.arange(height), np.arange(width), indexing="ij")
    parts = []
    for pos, n in ((t, n_t), (y, n_y), (x, n_x)):
        freq = ROPE_THETA ** (-np.arange(n, dtype=np.float64) / n)
        parts.append(pos.reshape(-1, 1).astype(np.float64) * freq[None, :])
    return np.concatenate(parts, axis=1)


def apply_rope(x: np.ndarray, angles: np.ndarray, n_heads: int) -> np.ndarray:
    """Rotate the channel pairs (2i, 2i+1) of every head by angles[:, i]:
    (a, b) -> (a cos - b sin, a sin + b cos).  angles: [rows, head_dim/2]."""
    r, d = x.shape
    xh = x.reshape(r, n_heads, d // n_heads // 2, 2)
    c, s_ = np.cos(angles)[:, None, :], np.sin(angles)[:, None, :]
    a, b = xh[..., 0], xh[..., 1]
    return np.stack([a * c - b * s_, a * s_ + b * c], axis=-1).reshape(r, d)


class BlockExt:
    """What the modulated block needs beyond the plain one: which parts are on, the
    number of text rows (they take the text-stream modulation and no rotation) and
    the rotation angles of the video tokens."""

    def __init__(self, cfg):
        self.flags = int(getattr(cfg, "block_flags", 0))
        self.n_text = cfg.n_text
        self.n_heads = cfg.n_heads
        self.angles = (rope_angles(cfg.frames, cfg.height, cfg.width, cfg.head_dim)
                       if self.flags & BLOCK_ROPE else None)

    def ln(self, x_rows, rows, w, which, eps):
        u = layer_norm(x_rows, w[f"ln{which}_g"], w[f"ln{which}_b"], eps)
        if self.flags & BLOCK_ADALN:
            u = (u * (1.0 + stream_vector(w["mod"], f"scale{which}", rows, self.n_text))
                 + stream_vector(w["mod"], f"shift{which}", rows, self.n_text))
        return u

    def gate(self, g_rows, rows, w, which):
        if self.flags & BLOCK_ADALN:
            return g_rows * stream_vector(w["mod"], f"gate{which}", rows, self.n_text)
        return g_rows

    def qk(self, q, k, rows, w):
        if self.flags & BLOCK_QKNORM:
            q = head_layer_norm(q, w["qn_g"], w["qn_b"], self.n_heads)
            k = head_layer_norm(k, w["kn_g"], w["kn_b"], self.n_heads)
        if self.flags & BLOCK_ROPE:
            rows = np.asarray(rows)
            vid = rows >= self.n_text
            if vid.any():
                ang = self.angles[rows[vid] - self.n_text]
                q, k = q.copy(), k.copy()
                q[vid] = apply_rope(q[vid], ang, self.n_heads)
                k[vid] = apply_rope(k[vid], ang, self.n_heads)
        return q, k


def refresh_rows_ext(x: np.ndarray, w, cache: "LayerCache", idx: np.ndarray, ext: BlockExt, eps: float) -> None:
    """Eq. 3 on rows idx with the modulated block; updates the cache in place.
    Cached features are what is added to the stream, i.e. after the gate."""
    d = x.shape[1]
    u = ext.ln(x[idx], idx, w, 1, eps)
    qkv = linear(u, w["w_qkv"], w["b_qkv"])
    q, k = ext.qk(qkv[:, :d], qkv[:, d:2 * d], idx, w)
    cache.k[idx] = k
    cache.v[idx] = qkv[:, 2 * d:]
    g_attn = ext.gate(linear(attention(q, cache.k, cache.v, ext.n_heads), w["w_o"], w["b_o"]), idx, w, 1)
    cache.g_attn[idx] = g_attn
    a = x[idx] + g_attn
    cache.g_ffn[idx] = ext.gate(ffn(ext.ln(a, idx, w, 2, eps), w), idx, w, 2)


class LayerCache:
    """Cached features of one layer: G of the attention branch and of the FFN
    branch for all N rows (the paper's G on video rows, H on text rows), the
    previous full-step generation of both (deep layers), and K, V of every row
    (shallow layers)."""

    def __init__(self):
        self.g_attn: Optional[np.ndarray] = None
        self.g_ffn: Optional[np.ndarray] = None
        self.g_attn_prev: Optional[np.ndarray] = None
        self.g_ffn_prev: Optional[np.ndarray] = None
        self.k: Optional[np.ndarray] = None
        self.v: Optional[np.ndarray] = None
        self.n_fills = 0


def block_forward(x: np.ndarray, w: Dict[str, np.ndarray], n_heads: int, eps: float):
    """Eq. 2 on all rows.  Returns (y, g_attn, g_ffn, k, v)."""
    d = x.shape[1]
    u = layer_norm(x, w["ln1_g"], w["ln1_b"], eps)
    qkv = linear(u, w["w_qkv"], w["b_qkv"])
    q, k, v = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
    g_attn = linear(attention(q, k, v, n_heads), w["w_o"], w["b_o"])
    a = x + g_attn
    g_ffn = ffn(layer_norm(a, w["ln2_g"], w["ln2_b"], eps), w)
    return a + g_ffn, g_attn, g_ffn, k, v


def full_layer(x: np.ndarray, w, cache: LayerCache, n_heads: int, eps: float,
               keep_kv: bool, keep_prev: bool) -> np.ndarray:
    """Alg. 1, initial caching of one layer: compute everything, fill the cache."""
    y, g_attn, g_ffn, k, v = block_forward(x, w, n_heads, eps)
    if keep_prev:
        cache.g_attn_prev, cache.g_ffn_prev = cache.g_attn, cache.g_ffn
    cache.g_attn, cache.g_ffn = g_attn, g_ffn
    if keep_kv:
        cache.k, cache.v = k, v
    cache.n_fills += 1
    return y


def refresh_layer(x: np.ndarray, w, cache: LayerCache, idx: np.ndarray,
                  n_heads: int, eps: float) -> np.ndarray:
    """Eq. 3 / Alg. 1 (l < K): refresh rows idx, reuse the cache for all others."""
    d = x.shape[1]
    idx = np.asarray(idx, dtype=np.int64)
    if len(idx):
        u = layer_norm(x[idx], w["ln1_g"], w["ln1_b"], eps)
        qkv = linear(u, w["w_qkv"], w["b_qkv"])
        q, k, v = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
        cache.k[idx] = k
        cache.v[idx] = v
        g_attn = linear(attention(q, cache.k, cache.v, n_heads), w["w_o"], w["b_o"])
        cache.g_attn[idx] = g_attn
        a = x[idx] + g_attn
        cache.g_ffn[idx] = ffn(layer_norm(a, w["ln2_g"], w["ln2_b"], eps), w)
    return x + cache.g_attn + cache.g_ffn


def extrapolated(cur: np.ndarray, prev: Optional[np.ndarray], k: int, interval: int) -> np.ndarray:
    """Eq. 5: G_{t-k} = G_t + (G_t - G_{t+M}) * k / M; Delta = 0 while no G_{t+M} exists."""
    if prev is None:
        return cur.copy()
    return cur + (cur - prev) * (k / interval)


def extrapolate_layer(x: np.ndarray, cache: LayerCache, k: int, interval: int) -> np.ndarray:
    """Alg. 1 (l >= K): both sub-modules' features are extrapolated, then added."""
    return (x + extrapolated(cache.g_attn, cache.g_attn_prev, k, interval)
            + extrapolated(cache.g_ffn, cache.g_ffn_prev, k, interval))


# ----------------------------------------------------------------------------
# the step (Alg. 1 outer loops)
# ----------------------------------------------------------------------------

class HeroOracle:
    """State of one video's denoising run: per-layer caches, token ages, schedule."""

    def __init__(self, cfg, weights: List[Dict[str, np.ndarray]], dtype=np.float64):
        self.cfg = cfg
        self.dtype = dtype
        self.w = [_cast_weights(w, dtype) for w in weights]
        self.reset()

    def reset(self):
        self.caches = [LayerCache() for _ in range(self.cfg.n_layers)]
        self.ages = np.zeros(self.cfg.n_video, dtype=np.int32)
        self.n_full = 0
        self.last_full = -1
        self.last_idx: Optional[np.ndarray] = None

    def is_full_step(self, step: int) -> bool:
        return step % self.cfg.interval == 0

    def _ext(self):
        if not hasattr(self, "_ext_cached"):
            self._ext_cached = BlockExt(self.cfg) if getattr(self.cfg, "block_flags", 0) else None
        return self._ext_cached

    def full_layer(self, layer: int, x: np.ndarray) -> np.ndarray:
        c = self.cfg
        shallow = layer < c.n_shallow
        if self._ext() is not None:
            # the modulated block on all rows: a refresh of every row into a fresh cache
            x = np.asarray(x, self.dtype)
            cache, n = self.caches[layer], x.shape[0]
            if not shallow:
                cache.g_attn_prev, cache.g_ffn_prev = cache.g_attn, cache.g_ffn
            cache.g_attn, cache.g_ffn = np.zeros_like(x), np.zeros_like(x)
            cache.k, cache.v = np.zeros_like(x), np.zeros_like(x)
            refresh_rows_ext(x, self.w[layer], cache, np.arange(n), self._ext(), c.ln_eps)
            cache.n_fills += 1
            return x + cache.g_attn + cache.g_ffn
        return full_layer(np.asarray(x, self.dtype), self.w[layer], self.caches[layer],
                          c.n_heads, c.ln_eps, keep_kv=shallow, keep_prev=not shallow)

    def refresh_layer(self, layer: int, x: np.ndarray, idx: np.ndarray) -> np.ndarray:
        c = self.cfg
        if self._ext() is not None:
            x = np.asarray(x, self.dtype)
            idx = np.asarray(idx, dtype=np.int64)
            cache = self.caches[layer]
            if len(idx):
                refresh_rows_ext(x, self.w[layer], cache, idx, self._ext(), c.ln_eps)
            return x + cache.g_attn + cache.g_ffn
        return refresh_layer(np.asarray(x, self.dtype), self.w[layer], self.caches[layer],
                             idx, c.n_heads, c.ln_eps)

    def extrapolate_layer(self, layer: int, x: np.ndarray, k: int) -> np.ndarray:
        return extrapolate_layer(np.asarray(x, self.dtype), self.caches[layer], k, self.cfg.interval)

    def select(self, step: int) -> np.ndarray:
        idx, self.ages = select(self.ages, self.cfg, step)
        self.last_idx = idx
        return idx

    def step(self, x: np.ndarray, step: int) -> np.ndarray:
        c = self.cfg
        x = np.asarray(x, self.dtype)
        if self.is_full_step(step):
            for l in range(c.n_layers):
                x = self.full_layer(l, x)
            self.ages[:] = 0
            self.n_full += 1
            self.last_full = step
            self.last_idx = None
            return x
        if self.n_full == 0:
            raise RuntimeError("cached step before any full step")
        k = step - self.last_full
        idx = self.select(step)
        for l in range(c.n_layers):
            if l < c.n_shallow:
                x = self.refresh_layer(l, x, idx)
            else:
                x = self.extrapolate_layer(l, x, k)
        return x


# ----------------------------------------------------------------------------
# stability score (Sec. 3.2, hierarchical feature analysis)
# ----------------------------------------------------------------------------

def second_difference_variance(features: List[np.ndarray]) -> float:
    """Variance of the second-order temporal differences of one layer's features.

    features: the layer's feature at T >= 3 consecutive (full) steps, equal shapes.
    D_t = F_{t+1} - 2 F_t + F_{t-1} for t = 1..T-2; the variance is taken over all
    elements of all D_t together (population variance, float64)."""
    f = [np.asarray(a, dtype=np.float64) for a in features]
    if len(f) < 3:
        raise ValueError("need at least three steps")
    d = np.concatenate([(f[t + 1] - 2.0 * f[t] + f[t - 1]).ravel() for t in range(1, len(f) - 1)])
    return float(np.mean((d - d.mean()) ** 2))


def stability_scores(variances) -> np.ndarray:
    """Per-layer variances -> scores in [0, 1], higher = more stable: min-max
    normalisation, inverted (the steadiest layer scores 1, the most variable 0;
    all equal -> all 1)."""
    v = np.asarray(variances, dtype=np.float64)
    lo, hi = v.min(), v.max()
    if hi == lo:
        return np.ones_like(v)
    return 1.0 - (v - lo) / (hi - lo)


# ----------------------------------------------------------------------------
# cost model (what the paper's FLOPs columns count), used by the Table 3/4 pin
# ----------------------------------------------------------------------------

def layer_flops(n_rows: int, n_keys: int, d: int, ffn_dim: int) -> float:
    """Matmul FLOPs of one block on n_rows queries against n_keys keys:
    QKV 6 r d^2, out-proj 2 r d^2, FFN 4 r d d_ff, attention 4 r N d."""
    return 8.0 * n_rows * d * d + 4.0 * n_rows * d * ffn_dim + 4.0 * n_rows * n_keys * d


def schedule_flops(cfg, n_steps: int, refreshed_rows: Optional[int] = None) -> float:
    """FLOPs of a whole schedule under Alg. 1: full steps run every layer on all
    rows; cached steps run the shallow layers on the refreshed rows against all
    keys; extrapolated layers cost nothing."""
    n = cfg.n_tokens
    full = cfg.n_layers * layer_flops(n, n, cfg.hidden, cfg.ffn_dim)
    if refreshed_rows is None:
        refreshed_rows = sum(tokens_per_patch(cfg.ratio, hh * ww) for (_, _, _, hh, ww) in
                             patch_list(cfg.frames, cfg.height, cfg.width, cfg.patch_h, cfg.patch_w))
    cached = cfg.n_shallow * layer_flops(refreshed_rows, n, cfg.hidden, cfg.ffn_dim)
    n_full = sum(1 for s in range(n_steps) if s % cfg.interval == 0)
    return n_full * full + (n_steps - n_full) * cached
