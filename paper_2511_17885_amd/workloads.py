"""Seeded synthetic workloads for the MoE-layer prefill path.

This module only draws random inputs and converts number formats.  It holds none
of the method's arithmetic (no softmax, top-k, scoring, FFN): both the CPU
oracle's tests and the HIP path's tests/bench take their inputs from here so that
the two sides see the same bytes.

The inputs stand in for the paper's workloads (high-resolution multi-tile images
through DeepSeek-VL2 / InternVL3.5, Sec. 2.1 and App. A): long runs of visual
tokens followed by a short text prompt, with neighbouring visual tokens close to
each other (the observation behind Fig. 1), and a skewed expert load.

Sequence layout follows Sec. 3.2.1: every sequence is [T_v, T_t], visual tokens
first.  All arrays are numpy; floating point arrays are float32 and, for the
bf16 workloads, already hold only bf16-representable values.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional, Sequence

import numpy as np

F32 = "f32"
BF16 = "bf16"


# --------------------------------------------------------------------------
# number-format helpers (no method arithmetic)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even) and return the raw 16-bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen raw bfloat16 bit patterns to float32 (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_dtype(a: np.ndarray, dtype: str) -> np.ndarray:
    """Return float32 values representable in `dtype` (identity for f32)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == BF16:
        return bf16_bits_to_f32(f32_to_bf16_bits(a))
    return a


# --------------------------------------------------------------------------
# workload container
# --------------------------------------------------------------------------
@dataclasses.dataclass
class LayerWeights:
    router_w: np.ndarray                 # [E, d]
    router_bias: Optional[np.ndarray]    # [E] float32 or None
    w_gate: np.ndarray                   # [E, F, d]
    w_up: np.ndarray                     # [E, F, d]
    w_down: np.ndarray                   # [E, d, F]
    ws_gate: Optional[np.ndarray]        # [N_s, F_s, d] or None
    ws_up: Optional[np.ndarray]
    ws_down: Optional[np.ndarray]        # [N_s, d, F_s]


@dataclasses.dataclass
class Workload:
    name: str
    dtype: str            # "f32" | "bf16"
    d: int                # hidden size H
    E: int                # routed experts
    F: int                # expert intermediate size S_m
    n_shared: int
    F_shared: int
    k_text: int
    k_visual: int
    retention: float
    window: int
    x: np.ndarray         # [T, d]
    is_visual: np.ndarray  # [T] uint8
    cu_seqlens: np.ndarray  # [B+1] int32
    layers: Sequence[LayerWeights]   # a list, or LazyLayers for the stack workloads
    # per-layer (k_text, k_visual) and the layer after which pruning runs (stack workloads)
    k_schedule: Optional[List[Sequence[int]]] = None
    prune_after_layer: Optional[int] = None

    @property
    def T(self) -> int:
        return int(self.x.shape[0])

    @property
    def B(self) -> int:
        return int(self.cu_seqlens.shape[0] - 1)

    @property
    def weights(self) -> LayerWeights:
        return self.layers[0]


class LazyLayers:
    """The layers of a stack workload, each drawn on demand from a random stream of its own, so that a
    12-layer stack of full-size layers (2.3 GB of fp32 per layer on the host) never has to exist at
    once.  Indexing draws the layer again every time: callers keep what they need."""

    def __init__(self, n_layers, draw):
        self._n, self._draw = int(n_layers), draw

    def __len__(self):
        return self._n

    def __getitem__(self, l):
        if isinstance(l, slice):
            return [self[i] for i in range(*l.indices(self._n))]
        if l < 0:
            l += self._n
        if not 0 <= l < self._n:
            raise IndexError(l)
        return self._draw(l)

    def __iter__(self):
        return (self._draw(l) for l in range(self._n))


def _round_bf16_inplace(a: np.ndarray) -> np.ndarray:
    """round_to_dtype(a, BF16) without temporaries of the array's size (same values)."""
    u = a.view(np.uint32)
    bias = u >> np.uint32(16)
    bias &= np.uint32(1)
    bias += np.uint32(0x7FFF)
    u += bias
    u &= np.uint32(0xFFFF0000)
    return a


def _normal(rng: np.random.Generator, shape, std: float, dtype: str) -> np.ndarray:
    a = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return _round_bf16_inplace(a) if dtype == BF16 else a


def draw_layer_weights(rng, d, E, F, n_shared, F_shared, bias_std, dtype, w_std=0.02) -> LayerWeights:
    router_w = _normal(rng, (E, d), w_std, dtype)
    router_bias = None
    if bias_std > 0.0:
        router_bias = (rng.standard_normal(E, dtype=np.float32) * np.float32(bias_std)).astype(np.float32)
    w_gate = _normal(rng, (E, F, d), w_std, dtype)
    w_up = _normal(rng, (E, F, d), w_std, dtype)
    w_down = _normal(rng, (E, d, F), w_std, dtype)
    ws_gate = ws_up = ws_down = None
    if n_shared > 0:
        ws_gate = _normal(rng, (n_shared, F_shared, d), w_std, dtype)
        ws_up = _normal(rng, (n_shared, F_shared, d), w_std, dtype)
        ws_down = _normal(rng, (n_shared, d, F_shared), w_std, dtype)
    return LayerWeights(router_w, router_bias, w_gate, w_up, w_down, ws_gate, ws_up, ws_down)


def draw_layer_weights_parallel(entropy, d, E, F, n_shared, F_shared, bias_std, dtype, w_std=0.02,
                                down_std=None) -> LayerWeights:
    """The same tensors as draw_layer_weights, each from a stream of its own (entropy + [tensor index]),
    so that the large ones can be drawn by separate threads.  down_std: standard deviation of the down
    projections (default w_std)."""
    import concurrent.futures as cf

    def stream(j):
        return np.random.Generator(np.random.PCG64(list(entropy) + [j]))

    shapes = [(E, F, d), (E, F, d), (E, d, F)]
    if n_shared > 0:
        shapes += [(n_shared, F_shared, d), (n_shared, F_shared, d), (n_shared, d, F_shared)]
    down_std = w_std if down_std is None else down_std
    with cf.ThreadPoolExecutor(max_workers=3) as ex:
        big = list(ex.map(lambda js: _normal(stream(2 + js[0]), js[1], down_std if js[0] % 3 == 2 else w_std, dtype),
                          enumerate(shapes)))
    router_w = _normal(stream(0), (E, d), w_std, dtype)
    router_bias = None
    if bias_std > 0.0:
        router_bias = (stream(1).standard_normal(E, dtype=np.float32) * np.float32(bias_std)).astype(np.float32)
    return LayerWeights(router_w, router_bias, *big, *([None] * (6 - len(big))))


def draw_visual_mixture(rng, n_tokens, d, n_components, sigma, max_run=16) -> np.ndarray:
    """Visual tokens from a Gaussian mixture with run-coherent component assignment.

    Component centres ~ N(0, I); runs of 1..max_run consecutive tokens share one
    component (chosen uniformly), each token = centre + sigma * N(0, I).  Runs make
    neighbouring tokens redundant, as adjacent image patches are.
    """
    centres = rng.standard_normal((n_components, d), dtype=np.float32)
    comp = np.empty(n_tokens, dtype=np.int64)
    pos = 0
    while pos < n_tokens:
        run = int(rng.integers(1, max_run + 1))
        c = int(rng.integers(0, n_components))
        comp[pos:pos + run] = c
        pos += run
    noise = rng.standard_normal((n_tokens, d), dtype=np.float32)
    noise *= np.float32(sigma)
    return centres[comp] + noise


def _sequence(rng, n_visual, n_text, d, n_components, sigma, tile=None):
    """One [T_v, T_t] sequence.  `tile` = tokens per image tile, each tile with its own mixture."""
    parts = []
    if n_visual > 0:
        if tile is None:
            parts.append(draw_visual_mixture(rng, n_visual, d, n_components, sigma))
        else:
            done = 0
            while done < n_visual:
                n = min(tile, n_visual - done)
                parts.append(draw_visual_mixture(rng, n, d, n_components, sigma))
                done += n
    if n_text > 0:
        parts.append(rng.standard_normal((n_text, d), dtype=np.float32))
    x = np.concatenate(parts, axis=0) if parts else np.zeros((0, d), np.float32)
    mask = np.concatenate([np.ones(n_visual, np.uint8), np.zeros(n_text, np.uint8)])
    return x, mask


def make_workload(name: str, *, seed: int, dtype: str, d: int, E: int, F: int,
                  n_shared: int = 0, F_shared: Optional[int] = None,
                  k_text: int, k_visual: int, retention: float, window: int,
                  visual_lens: Sequence[int], text_lens: Sequence[int],
                  n_components: int = 0, sigma: float = 0.3, tile: Optional[int] = None,
                  bias_std: float = 0.0, n_layers: int = 1,
                  k_schedule=None, prune_after_layer=None, independent_layers: bool = False,
                  down_std: Optional[float] = None) -> Workload:
    """Draw weights first (layer by layer), then activations, from one PCG64 stream.
    independent_layers (stack workloads): the activations come from the stream seeded [seed, 0] and
    layer l from the stream seeded [seed, 1, l], drawn on demand (LazyLayers)."""
    F_shared = F if F_shared is None else F_shared
    if independent_layers:
        rng = np.random.Generator(np.random.PCG64([seed, 0]))
        layers = LazyLayers(n_layers, lambda l: draw_layer_weights_parallel(
            [seed, 1, l], d, E, F, n_shared, F_shared, bias_std, dtype, down_std=down_std))
    else:
        rng = np.random.Generator(np.random.PCG64(seed))
        layers = [draw_layer_weights(rng, d, E, F, n_shared, F_shared, bias_std, dtype)
                  for _ in range(n_layers)]
    xs, masks, cu = [], [], [0]
    for nv, nt in zip(visual_lens, text_lens):
        if n_components > 0:
            x, m = _sequence(rng, nv, nt, d, n_components, sigma, tile)
        else:
            x = rng.standard_normal((nv + nt, d), dtype=np.float32)
            m = np.concatenate([np.ones(nv, np.uint8), np.zeros(nt, np.uint8)])
        xs.append(x)
        masks.append(m)
        cu.append(cu[-1] + nv + nt)
    x = round_to_dtype(np.concatenate(xs, axis=0), dtype)
    return Workload(name=name, dtype=dtype, d=d, E=E, F=F, n_shared=n_shared, F_shared=F_shared,
                    k_text=k_text, k_visual=k_visual, retention=retention, window=window,
                    x=x, is_visual=np.concatenate(masks).astype(np.uint8),
                    cu_seqlens=np.asarray(cu, dtype=np.int32), layers=layers,
                    k_schedule=k_schedule, prune_after_layer=prune_after_layer)


# --------------------------------------------------------------------------
# the five benchmark configurations (and scaled-down variants of them)
# --------------------------------------------------------------------------
def config1() -> Workload:
    """Tiny fp32 layer: 48 visual + 16 text, d=128, 8 experts of 256, top-2/top-1, keep 75 %."""
    return make_workload("c1_tiny_fp32", seed=0, dtype=F32, d=128, E=8, F=256,
                         k_text=2, k_visual=1, retention=0.75, window=4,
                         visual_lens=[48], text_lens=[16])


def config2(scale: float = 1.0) -> Workload:
    """DeepSeek-VL2-Tiny-like: 1536 visual (96-component mixture) + 64 text, d=1280,
    64 experts of 896 + 2 shared, top-6/top-3, router bias N(0,1), keep 50 %, W=3."""
    nv, nt = int(round(1536 * scale)), max(1, int(round(64 * scale)))
    return make_workload("c2_dsvl2_tiny", seed=1, dtype=BF16, d=1280, E=64, F=896, n_shared=2,
                         k_text=6, k_visual=3, retention=0.5, window=3,
                         visual_lens=[nv], text_lens=[nt], n_components=96, bias_std=1.0)


def config3(retention: float = 0.5, k_visual: int = 3, scale: float = 1.0) -> Workload:
    """DeepSeek-VL2-Small-like: 3840 visual (192 components) + 256 text, d=2048,
    64 experts of 1408 + 2 shared, top-6/top-3, W=3; retention swept."""
    nv, nt = int(round(3840 * scale)), max(1, int(round(256 * scale)))
    return make_workload("c3_dsvl2_small", seed=2, dtype=BF16, d=2048, E=64, F=1408, n_shared=2,
                         k_text=6, k_visual=k_visual, retention=retention, window=3,
                         visual_lens=[nv], text_lens=[nt], n_components=192, bias_std=1.0)


def config4(scale: float = 1.0) -> Workload:
    """InternVL3.5-MoE-like: 31 tiles x 256 visual (64-component mixture per tile) + 256 text,
    d=2048, 128 experts of 768, top-8/top-4, router bias N(0,1.5), keep 50 %, W=5."""
    tiles = max(1, int(round(31 * scale)))
    nt = max(1, int(round(256 * scale)))
    return make_workload("c4_internvl35", seed=3, dtype=BF16, d=2048, E=128, F=768,
                         k_text=8, k_visual=4, retention=0.5, window=5,
                         visual_lens=[tiles * 256], text_lens=[nt], n_components=64, tile=256,
                         bias_std=1.5)


def config5_lengths(seed: int = 4, n_seqs: int = 8, lo: int = 1024, hi: int = 6400, step: int = 256):
    """Visual lengths of the ragged batch: uniform over {lo, lo+step, ..., hi}."""
    rng = np.random.Generator(np.random.PCG64(seed + 1000))
    choices = np.arange(lo, hi + 1, step)
    return [int(v) for v in rng.choice(choices, size=n_seqs)]


def config5(n_layers: int = 12, d: int = 2048, E: int = 64, F: int = 1408, n_shared: int = 2,
            len_div: int = 1, n_seqs: int = 8, text_len: int = 128, dtype: str = BF16) -> Workload:
    """Ragged batched prefill: 8 packed sequences (visual 1024..6400 step 256, +128 text),
    a 12-layer stack of config-3-shaped layers with x <- x + MoE(x); top-6/top-6 in layers
    0-1, top-6/top-3 from layer 2; pruning to 50 % once, after layer 2, per sequence.
    `len_div`, `d`, `F`, `n_layers` shrink it for tests the oracle must finish quickly.
    The stack has no normalisation layers (attention is an identity residual), and the SwiGLU expert
    term grows with the square of its input's scale, so with N(0, 0.02) everywhere the residual stream
    of twelve full-size layers diverges until fp32 overflows.  The down projections of the stack's
    layers are therefore drawn with standard deviation 0.02 / sqrt(2 * 12), the usual scaling of
    residual-branch output weights with depth, which keeps x at O(1) through the stack."""
    lens = [max(1, v // len_div) for v in config5_lengths(n_seqs=n_seqs)]
    sched = [(6, 6) if l < 2 else (6, 3) for l in range(n_layers)]
    return make_workload("c5_ragged_stack", seed=4, dtype=dtype, d=d, E=E, F=F, n_shared=n_shared,
                         k_text=6, k_visual=3, retention=0.5, window=3,
                         visual_lens=lens, text_lens=[max(1, text_len // len_div)] * n_seqs,
                         n_components=192, bias_std=1.0, n_layers=n_layers,
                         k_schedule=sched, prune_after_layer=2, independent_layers=True,
                         down_std=0.02 / float(np.sqrt(24.0)))


def small_random(seed: int, *, T_v: Sequence[int], T_t: Sequence[int], d: int, E: int, F: int,
                 k_text: int, k_visual: int, retention: float, window: int, dtype: str = F32,
                 n_shared: int = 0, F_shared: Optional[int] = None, bias_std: float = 0.0,
                 n_components: int = 0, interleave: bool = False) -> Workload:
    """Small randomised shapes for edge-case parity tests.  `interleave` shuffles the modality
    mask inside each sequence so visual tokens are not contiguous."""
    wl = make_workload(f"rand{seed}", seed=seed, dtype=dtype, d=d, E=E, F=F, n_shared=n_shared,
                       F_shared=F_shared, k_text=k_text, k_visual=k_visual, retention=retention,
                       window=window, visual_lens=T_v, text_lens=T_t, n_components=n_components,
                       bias_std=bias_std)
    if interleave:
        rng = np.random.Generator(np.random.PCG64(seed + 77))
        m = wl.is_visual.copy()
        for b in range(wl.B):
            s, e = int(wl.cu_seqlens[b]), int(wl.cu_seqlens[b + 1])
            seg = m[s:e].copy()
            rng.shuffle(seg)
            m[s:e] = seg
        wl.is_visual = m
    return wl


CONFIGS: Dict[str, object] = {
    "c1": config1, "c2": config2, "c3": config3, "c4": config4, "c5": config5,
}
